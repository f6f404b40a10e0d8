"""GPU parity of one whole decoder layer (attention half, then MLP half; seven fused multi-LoRA projections) against
the fp64 oracle on the same seeded bf16 inputs; the results must hold the tolerance against the plain fp64 oracle
and against the oracle that rounds the tensors the layer keeps in memory between its kernels."""
import numpy as np
import pytest

from oracle import layer_oracle as ly
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
HD = 128


LAYER_CASES = [(256, 640, 4, 2, [8, 0, 24, 3], [300, 0, 513, 70], [2.0, 1.0, 0.5, 4.0], [0, 100, 300, 301, 600, 813, 883]),
               (128, 384, 2, 2, [1, 130], [129, 260], [1.5, 1.5], [0, 129, 130, 389]),
               (512, 1024, 8, 2, [32], [515], [1.0], [0, 515])]


@pytest.mark.parametrize("case", LAYER_CASES, ids=["four_jobs", "odd_ranks", "one_job_long_seq"])
def test_decoder_layer_matches_oracle(case):
    import torch
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv, ranks, tokens, scales, seq = case
    seq = np.array(seq, dtype=np.int64)
    eps, base = 1e-5, 10000.0
    rng = np.random.default_rng(8)
    f = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32))
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    layers = {n: (f(rng.normal(size=(i, o)) / np.sqrt(i)), [f(rng.uniform(-1, 1, size=(i, r)) / np.sqrt(i)) for r in ranks],
                  [f(0.05 * rng.normal(size=(r, o))) for r in ranks]) for n, (i, o) in shapes.items()}
    X, dOut = f(rng.normal(size=(T, d))), f(rng.normal(size=(T, d)))
    g_attn, g_mlp = f(1.0 + 0.1 * rng.normal(size=d)), f(1.0 + 0.1 * rng.normal(size=d))
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=torch.bfloat16).contiguous()
    tl = {n: (up(W), [up(a) for a in A], [up(b) for b in B]) for n, (W, A, B) in layers.items()}
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, base, ranks, off, scales, seq, up(X), up(g_attn), up(g_mlp), eps, tl)
    Out = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    dX = torch.full_like(Out, float("nan"))
    grads = layer.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    layer.fwd(Out)
    layer.bwd(up(dOut), dX, grads)
    torch.cuda.synchronize()
    attn = (g_attn, eps, {n: layers[n] for n in ("q", "k", "v", "o")})
    mlp = (g_mlp, eps, {n: layers[n] for n in ("gate", "up", "down")})
    args = (attn, mlp, scales, off, seq, Hq, Hkv, HD, base)

    def oracle(store):
        out_r, _ = ly.forward(X, *args, store)
        dX_r, g_r = ly.backward(X, *args, dOut, store)
        return out_r, dX_r, g_r
    # two blocks chained: each block's error budget (see the block tests) adds
    res = pu.block_report("decoder layer", Out, dX, grads, oracle, 2 * pu.BF16_TOL, pu.bf16_store, rms_floor_on_acts=True)
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"worst error / tolerance ratios {res}"


def test_decoder_layer_without_tokens_gives_zero_gradients():
    import torch
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv = 256, 384, 2, 1
    ranks = [4, 8]
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    rn = lambda *sh: torch.randn(*sh, device="cuda", generator=g).to(torch.bfloat16)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    tl = {n: (rn(i, o), [rn(i, r) for r in ranks], [rn(r, o) for r in ranks]) for n, (i, o) in shapes.items()}
    X = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    gamma = torch.ones(d, dtype=torch.bfloat16, device="cuda")
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, 10000.0, ranks, [0, 0, 0], [1.0, 2.0], [0], X, gamma, gamma, 1e-5, tl)
    grads = layer.new_grads()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            t.fill_(float("nan"))
    layer.fwd(X)
    layer.bwd(X, X, grads)
    torch.cuda.synchronize()
    for n in grads:
        for t in grads[n][0] + grads[n][1]:
            assert float(t.abs().max()) == 0.0, n


def test_decoder_layer_training_steps_follow_the_oracle():
    """Four steps of forward, backward and AdamW on all 7 x J adapter pairs of one decoder layer (regression onto a
    fixed target): the loss falls, and its trajectory matches the same loop run with the oracles in float64 (with the
    bf16 storage points of the GPU path)."""
    import torch
    from oracle import adamw_oracle as adw
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv = 256, 384, 2, 1
    ranks, tokens, scales = [8, 4], [96, 64], [2.0, 1.0]
    seq = np.array([0, 96, 130, 160], dtype=np.int64)
    eps, base, lr, steps = 1e-5, 10000.0, 2e-3, 4
    rng = np.random.default_rng(31)
    f = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32))
    T = sum(tokens)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    names = list(shapes)
    W = {n: f(rng.normal(size=s) / np.sqrt(s[0])) for n, s in shapes.items()}
    A0 = {n: [rng.uniform(-1, 1, size=(s[0], r)).astype(np.float32) / np.float32(np.sqrt(s[0])) for r in ranks] for n, s in shapes.items()}
    B0 = {n: [(0.05 * rng.normal(size=(r, s[1]))).astype(np.float32) for r in ranks] for n, s in shapes.items()}
    X, target = f(rng.normal(size=(T, d))), f(rng.normal(size=(T, d)))
    gam = f(np.ones(d))
    store = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)

    # ---- oracle loop (fp64 masters; the layer reads their bf16 roundings) ----
    mA = {n: [a.astype(np.float64) for a in A0[n]] for n in names}
    mB = {n: [b.astype(np.float64) for b in B0[n]] for n in names}
    st = {n: [[np.zeros_like(a), np.zeros_like(a), np.zeros_like(b), np.zeros_like(b)] for a, b in zip(mA[n], mB[n])] for n in names}
    loss_r = []
    for t in range(1, steps + 1):
        layers = {n: (W[n], [store(a) for a in mA[n]], [store(b) for b in mB[n]]) for n in names}
        attn = (gam, eps, {n: layers[n] for n in ("q", "k", "v", "o")})
        mlp = (gam, eps, {n: layers[n] for n in ("gate", "up", "down")})
        args = (attn, mlp, scales, off, seq, Hq, Hkv, HD, base)
        out, _ = ly.forward(X, *args, store)
        diff = store(out) - target
        loss_r.append(0.5 * float(np.sum(diff * diff)))
        _, g = ly.backward(X, *args, store(diff), store)
        for n in names:
            for j in range(len(ranks)):
                mA[n][j], st[n][j][0], st[n][j][1] = adw.adamw_step(mA[n][j], g[n][0][j], st[n][j][0], st[n][j][1], t, lr)
                mB[n][j], st[n][j][2], st[n][j][3] = adw.adamw_step(mB[n][j], g[n][1][j], st[n][j][2], st[n][j][3], t, lr)

    # ---- GPU loop ----
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device="cuda", dtype=torch.bfloat16).contiguous()
    master = {n: ([torch.from_numpy(a.copy()).cuda() for a in A0[n]], [torch.from_numpy(b.copy()).cuda() for b in B0[n]]) for n in names}
    tl = {n: (up(W[n]), [m_.to(torch.bfloat16) for m_ in master[n][0]], [m_.to(torch.bfloat16) for m_ in master[n][1]]) for n in names}
    tX, tT = up(X), up(target)
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, base, ranks, off, scales, seq, tX, up(gam), up(gam), eps, tl)
    grads = layer.new_grads()
    params = [p_ for n in names for p_ in tl[n][1] + tl[n][2]]
    masters = [p_ for n in names for p_ in master[n][0] + master[n][1]]
    gl = [p_ for n in names for p_ in grads[n][0] + grads[n][1]]
    ms = [torch.zeros_like(p_) for p_ in masters]
    vs = [torch.zeros_like(p_) for p_ in masters]
    ows = torch.empty(tlora.tlora_adamw_workspace_bytes(len(params)), dtype=torch.uint8, device="cuda")
    Out, dX = torch.empty_like(tX), torch.empty_like(tX)
    loss_g = []
    for t in range(1, steps + 1):
        layer.fwd(Out)
        diff = (Out.float() - tT.float())
        loss_g.append(0.5 * float((diff.double() ** 2).sum()))
        layer.bwd(diff.to(torch.bfloat16), dX, grads)
        tens = [dict(param=p_.data_ptr(), master=w_.data_ptr(), grad=g_.data_ptr(), m=a_.data_ptr(), v=b_.data_ptr(),
                     n=p_.numel(), lr=lr, step=t) for p_, w_, g_, a_, b_ in zip(params, masters, gl, ms, vs)]
        tlora.tlora_adamw_step(tens, tlora.TLORA_BF16, ows.data_ptr(), ows.numel(), int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    print("loss oracle", [round(x, 2) for x in loss_r], "gpu", [round(x, 2) for x in loss_g])
    assert all(b < a for a, b in zip(loss_g[:-1], loss_g[1:])), loss_g
    assert all(abs(a - b) <= 1e-2 * b for a, b in zip(loss_g, loss_r)), (loss_g, loss_r)


def test_fused_decoder_layer_equals_each_job_alone():
    """Sec. 3.2: the shared super-model is functionally equivalent to training each job independently.  A layer run
    on two jobs together gives, for each job, exactly the outputs, input gradients and adapter gradients of that job
    run alone (same kernels, same order of every sum), bit for bit."""
    import torch
    from paper_2602_07263_amd import tlora
    d, dff, Hq, Hkv = 256, 384, 4, 2
    ranks, tokens, scales = [8, 20], [256, 300], [2.0, 0.5]        # job 0 ends on a row-tile boundary of the GEMM
    seqs = [[0, 100, 256], [0, 300]]                               # per job, relative to its first token
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    bf = torch.bfloat16
    rn = lambda *sh, std=1.0: (torch.randn(*sh, device="cuda", generator=g) * std).to(bf)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    W = {n: rn(i, o, std=i ** -0.5) for n, (i, o) in shapes.items()}
    A = {n: [rn(i, r, std=i ** -0.5) for r in ranks] for n, (i, o) in shapes.items()}
    B = {n: [rn(r, o, std=0.05) for r in ranks] for n, (i, o) in shapes.items()}
    T = sum(tokens)
    X, dOut = rn(T, d), rn(T, d)
    gam = torch.ones(d, device="cuda", dtype=bf)

    def run(jobs, rows):
        off = [0]
        seq = [0]
        for j in jobs:
            seq += [off[-1] + s for s in seqs[j][1:]]
            off.append(off[-1] + tokens[j])
        tl = {n: (W[n], [A[n][j] for j in jobs], [B[n][j] for j in jobs]) for n in shapes}
        Xs, dOs = X[rows].contiguous(), dOut[rows].contiguous()
        layer = tlora.DecoderLayer(d, dff, Hq, Hkv, 10000.0, [ranks[j] for j in jobs], off, [scales[j] for j in jobs], seq,
                                   Xs, gam, gam, 1e-5, tl)
        Out, dX, grads = torch.empty_like(Xs), torch.empty_like(Xs), layer.new_grads()
        layer.fwd(Out)
        layer.bwd(dOs, dX, grads)
        torch.cuda.synchronize()
        return Out, dX, grads
    Out_f, dX_f, g_f = run([0, 1], slice(0, T))
    lo = 0
    for j in (0, 1):
        rows = slice(lo, lo + tokens[j])
        Out_s, dX_s, g_s = run([j], rows)
        assert torch.equal(Out_f[rows].view(torch.int16), Out_s.view(torch.int16)), f"Out of job {j}"
        assert torch.equal(dX_f[rows].view(torch.int16), dX_s.view(torch.int16)), f"dX of job {j}"
        for n in shapes:
            assert torch.equal(g_f[n][0][j], g_s[n][0][0]) and torch.equal(g_f[n][1][j], g_s[n][1][0]), (n, j)
        lo += tokens[j]


def test_decoder_layer_at_bench_shape_sampled_jobs():
    """The decoder-layer leg's full shape (cfg3: 16 jobs, 83 968 tokens in sequences of 2048, d_model 4096, 32 / 8 heads,
    d_ff 12288), launched as bench.py launches it.  Jobs whose batch is a single sequence are independent of every
    other row of the batch, so the oracle can run them alone: their rows of Out and dX and their complete dA_j / dB_j
    of all seven projections are compared with the fused run."""
    import torch
    from paper_2602_07263_amd import tlora
    wl = wk.config(3)
    d, dff, Hq, Hkv, n = 4096, 12288, 32, 8, 2048
    T = wl.total_tokens
    g = torch.Generator(device="cuda"); g.manual_seed(0)
    bf = torch.bfloat16
    rn = lambda *shape, std=1.0: (torch.randn(*shape, device="cuda", generator=g) * std).to(bf)
    shapes = dict(q=(d, Hq * HD), k=(d, Hkv * HD), v=(d, Hkv * HD), o=(Hq * HD, d), gate=(d, dff), up=(d, dff), down=(dff, d))
    layers = {name: (rn(i, o, std=i ** -0.5), [((torch.rand(i, r, device="cuda", generator=g) * 2 - 1) / i ** 0.5).to(bf)
                                                for r in wl.ranks], [rn(r, o, std=0.01) for r in wl.ranks])
              for name, (i, o) in shapes.items()}
    X, dOut = rn(T, d), rn(T, d)
    gamma = torch.ones(d, device="cuda", dtype=bf)
    base, eps = 500000.0, 1e-5
    layer = tlora.DecoderLayer(d, dff, Hq, Hkv, base, wl.ranks, wl.offsets, wl.scales, list(range(0, T + 1, n)), X, gamma,
                               gamma, eps, layers)
    Out, dX, grads = torch.empty_like(X), torch.empty_like(X), layer.new_grads()
    layer.fwd(Out)
    layer.bwd(dOut, dX, grads)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Out.float()).all()) and bool(torch.isfinite(dX.float()).all())
    store = lambda a: wk.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)
    tol = 2 * pu.BF16_TOL                           # two blocks chained (see test_decoder_layer_matches_oracle)

    def ratio(got, ref):
        got = np.asarray(got, dtype=np.float64)
        assert np.all(np.isfinite(got))
        m = max(1.0, float(np.sqrt(np.mean(ref * ref))))
        return float(np.max(np.abs(got - ref) / (tol * (m + np.abs(ref)))))
    f64 = lambda t: t.double().cpu().numpy()
    worst = {}
    singles = [j for j, t in enumerate(wl.tokens) if t == n]
    for j in singles[-1:]:                           # the single-sequence job of the highest rank (64)
        rows = slice(wl.offsets[j], wl.offsets[j + 1])
        lay = {name: (f64(W), [f64(A[j])], [f64(B[j])]) for name, (W, A, B) in layers.items()}
        attn = (f64(gamma), eps, {k_: lay[k_] for k_ in ("q", "k", "v", "o")})
        mlp = (f64(gamma), eps, {k_: lay[k_] for k_ in ("gate", "up", "down")})
        args = (attn, mlp, [wl.scales[j]], [0, n], [0, n], Hq, Hkv, HD, base)
        out_r, _ = ly.forward(f64(X[rows]), *args, store)
        dX_r, g_r = ly.backward(f64(X[rows]), *args, f64(dOut[rows]), store)
        res = {"Out": ratio(f64(Out[rows]), out_r), "dX": ratio(f64(dX[rows]), dX_r)}
        for name in shapes:
            res["dA_" + name] = ratio(grads[name][0][j].cpu().numpy(), g_r[name][0][0])
            res["dB_" + name] = ratio(grads[name][1][j].cpu().numpy(), g_r[name][1][0])
        for k_, v_ in res.items():
            worst[k_] = max(worst.get(k_, 0.0), v_)
    print({k_: round(v_, 3) for k_, v_ in worst.items()})
    assert all(v_ <= 1.0 for v_ in worst.values()), worst
