"""GPU parity of the per-job AdamW step against the fp64 oracle, and a short training run of the fused layer
(forward, backward, optimizer step -- all through the C ABI) whose loss must go down."""
import numpy as np
import pytest

from oracle import adamw_oracle as ao
from paper_2602_07263_amd import workloads as wk

pytestmark = pytest.mark.gpu


def _bf16_round(x):
    return wk.round_to_bf16(np.asarray(x, dtype=np.float32))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_adamw_matches_oracle_elementwise(dtype):
    import torch
    from paper_2602_07263_amd import tlora
    rng = np.random.default_rng(12)
    sizes = [0, 1, 255, 4096, 4097, 70001, 8 * 12288]
    hyper = [dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, step=1),
             dict(lr=3e-4, beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1, step=17),
             dict(lr=1e-2, beta1=0.0, beta2=0.5, eps=1e-3, weight_decay=0.01, step=3)]
    dev = "cuda"
    tens, ref, keep = [], [], []
    for k, n in enumerate(sizes):
        h = hyper[k % len(hyper)]
        w = rng.normal(size=n).astype(np.float32)
        g = (rng.normal(size=n) * 10.0 ** rng.integers(-4, 1)).astype(np.float32)
        m = (0.1 * rng.normal(size=n)).astype(np.float32) if h["step"] > 1 else np.zeros(n, np.float32)
        v = (0.01 * rng.random(size=n)).astype(np.float32) if h["step"] > 1 else np.zeros(n, np.float32)
        t = {name: torch.from_numpy(a.copy()).to(dev) for name, a in dict(master=w, grad=g, m=m, v=v).items()}
        t["param"] = torch.empty(n, device=dev, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
        keep.append(t)
        tens.append(dict(param=t["param"].data_ptr() if n else 0, master=t["master"].data_ptr() if n else 0,
                         grad=t["grad"].data_ptr() if n else 0, m=t["m"].data_ptr() if n else 0,
                         v=t["v"].data_ptr() if n else 0, n=n, **h))
        ref.append(ao.adamw_step(w, g, m, v, h["step"], h["lr"], h["beta1"], h["beta2"], h["eps"], h["weight_decay"]))
    ws_bytes = tlora.tlora_adamw_workspace_bytes(len(tens))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    tlora.tlora_adamw_step(tens, tlora.TLORA_BF16 if dtype == "bf16" else tlora.TLORA_F32, ws.data_ptr(), ws_bytes,
                           int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    for t, (w_r, m_r, v_r), n in zip(keep, ref, sizes):
        w_g, m_g, v_g = (t[k].cpu().numpy().astype(np.float64) for k in ("master", "m", "v"))
        assert np.all(np.abs(w_g - w_r) <= 1e-5 * (1 + np.abs(w_r)))
        assert np.all(np.abs(m_g - m_r) <= 1e-6 * (1e-3 + np.abs(m_r)))
        assert np.all(np.abs(v_g - v_r) <= 1e-6 * (1e-6 + np.abs(v_r)))
        p_g = t["param"].float().cpu().numpy()
        # the tensor the layer reads is the master copy in the layer's dtype: same bits as rounding the GPU's own
        # master (the rounding decision is taken in fp32 on both sides)
        want = _bf16_round(t["master"].cpu().numpy()) if dtype == "bf16" else t["master"].cpu().numpy()
        assert np.array_equal(p_g, want)


def test_master_may_be_omitted_for_fp32_and_errors_are_reported():
    import ctypes
    import torch
    from paper_2602_07263_amd import tlora
    n = 1000
    rng = np.random.default_rng(1)
    w, g = rng.normal(size=n).astype(np.float32), rng.normal(size=n).astype(np.float32)
    p, gd = torch.from_numpy(w.copy()).cuda(), torch.from_numpy(g).cuda()
    m, v = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    t = dict(param=p.data_ptr(), master=0, grad=gd.data_ptr(), m=m.data_ptr(), v=v.data_ptr(), n=n, lr=1e-2, step=1)
    tlora.tlora_adamw_step([t], tlora.TLORA_F32, ws.data_ptr(), 256)
    torch.cuda.synchronize()
    w_r, _, _ = ao.adamw_step(w, g, np.zeros(n), np.zeros(n), 1, 1e-2)
    assert np.all(np.abs(p.cpu().numpy() - w_r) <= 1e-5 * (1 + np.abs(w_r)))
    with pytest.raises(tlora.TloraError):          # a bf16 tensor needs the fp32 master
        tlora.tlora_adamw_step([t], tlora.TLORA_BF16, ws.data_ptr(), 256)
    with pytest.raises(tlora.TloraError):          # step 0 has no bias correction
        tlora.tlora_adamw_step([dict(t, step=0)], tlora.TLORA_F32, ws.data_ptr(), 256)
    with pytest.raises(tlora.TloraError):
        tlora.tlora_adamw_step([t], tlora.TLORA_F32, 0, 0)


def test_a_few_training_steps_reduce_the_loss():
    """fwd -> bwd -> per-job AdamW, three jobs with their own learning rates, fixed batch and target."""
    import torch
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("train", "bf16", 256, 384, [8, 16, 4], [300, 500, 200], [2.0, 2.0, 2.0]), seed=6)
    lp = tlora.LayerProblem.from_numpy(p)
    rng = np.random.default_rng(7)
    target = torch.from_numpy(rng.normal(size=(lp.T, 384)).astype(np.float32)).cuda()
    Y, dX, dA, dB = lp.new_outputs()
    params = lp.A + lp.B
    grads = dA + dB
    master = [t.float().clone() for t in params]
    m = [torch.zeros_like(t) for t in master]
    v = [torch.zeros_like(t) for t in master]
    lrs = [3e-3, 1e-3, 2e-3] * 2
    ws_bytes = tlora.tlora_adamw_workspace_bytes(len(params))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    losses = []
    for step in range(1, 9):
        lp.fwd(Y)
        diff = Y.float() - target
        losses.append(float(0.5 * (diff * diff).sum()))
        dY = diff.to(torch.bfloat16)
        lp.bwd(dY, None, dA, dB, reuse_S=True)
        tens = [dict(param=q.data_ptr(), master=w.data_ptr(), grad=g.data_ptr(), m=a.data_ptr(), v=b.data_ptr(),
                     n=q.numel(), lr=lr, weight_decay=0.01, step=step)
                for q, w, g, a, b, lr in zip(params, master, grads, m, v, lrs)]
        tlora.tlora_adamw_step(tens, tlora.TLORA_BF16, ws.data_ptr(), ws_bytes)
    torch.cuda.synchronize()
    assert all(np.isfinite(losses)) and losses[-1] < losses[0] and losses[-1] < 0.999 * losses[0], losses
    assert all(b <= a * 1.0005 for a, b in zip(losses, losses[1:])), losses      # monotone up to bf16 noise
