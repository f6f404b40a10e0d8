"""GPU parity of the nano-batched execution (Sec. 3.3): the batch cut into N nano-batches, processed one after
the other through the C ABI, must give the oracle's result of the whole batch for every N (the nano-batch size is
a performance knob); dA_j / dB_j are accumulated over the nano-batches."""
import time

import numpy as np
import pytest

from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _assert_ok(res, label):
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"{label}: worst error / tolerance ratios {res}"


def _run_nano(p, n_nano, granule, flags=0, prefill=None):
    import torch
    from paper_2602_07263_amd import tlora
    lp = tlora.LayerProblem.from_numpy(p)
    tdt = torch.bfloat16 if p.dtype == "bf16" else torch.float32
    dY = torch.from_numpy(p.dY).to(device="cuda", dtype=tdt)
    Y, dX, dA, dB = lp.new_outputs()
    Y.fill_(float("nan")); dX.fill_(float("nan"))
    for t in dA + dB:
        t.fill_(float("nan") if prefill is None else prefill)
    lp.fwd_nano(n_nano, granule, Y)
    lp.bwd_nano(n_nano, granule, dY, dX, dA, dB, flags)
    torch.cuda.synchronize()
    return (Y.float().cpu().numpy(), dX.float().cpu().numpy(), [a.cpu().numpy() for a in dA],
            [b.cpu().numpy() for b in dB])


CASES = [
    ("bf16", 384, 640, [1, 12, 256, 40, 130], [300, 17, 700, 1, 520], [0.5, 2.0, 1.0, 4.0, 2.0]),
    ("f32", 96, 72, [3, 8, 0, 5], [40, 0, 33, 130], [2.0, 1.0, 2.0, 0.5]),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("n_nano,granule", [(1, 64), (2, 64), (5, 32), (9, 1), (64, 64)])
def test_results_do_not_depend_on_the_number_of_nano_batches(case, n_nano, granule):
    dtype, d_in, d_out, ranks, tokens, scales = case
    p = wk.generate(wk.custom("nano", dtype, d_in, d_out, ranks, tokens, scales), seed=5)
    Y, dX, dA, dB = _run_nano(p, n_nano, granule)
    _assert_ok(pu.compare(p, Y, dX, dA, dB), f"{dtype} N={n_nano} granule={granule}")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_accumulate_flag_adds_to_the_existing_gradients(dtype):
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("acc", dtype, 128, 192, [4, 16, 9], [100, 0, 260], [2.0, 2.0, 0.5]), seed=8)
    Y, dX, dA, dB = _run_nano(p, 3, 32, flags=tlora.TLORA_BWD_ACCUMULATE, prefill=1.5)
    res = pu.compare(p, Y, dX, [a - 1.5 for a in dA], [b - 1.5 for b in dB])
    _assert_ok(res, f"accumulate/{dtype}")
    # the job without tokens keeps what was there
    assert np.all(dA[1] == 1.5) and np.all(dB[1] == 1.5)
    # and the plain call accumulates too
    import torch
    lp = tlora.LayerProblem.from_numpy(p)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dYt = torch.from_numpy(p.dY).to(device="cuda", dtype=tdt)
    Yt, dXt, dAt, dBt = lp.new_outputs()
    for t in dAt + dBt:
        t.fill_(-2.0)
    lp.fwd(Yt)
    lp.bwd(dYt, dXt, dAt, dBt, reuse_S=True, flags=tlora.TLORA_BWD_ACCUMULATE)
    torch.cuda.synchronize()
    res = pu.compare(p, Yt.float().cpu().numpy(), dXt.float().cpu().numpy(), [a.cpu().numpy() + 2.0 for a in dAt],
                     [b.cpu().numpy() + 2.0 for b in dBt])
    _assert_ok(res, f"accumulate plain/{dtype}")


def test_reuse_of_the_transposed_weight():
    """A second backward with TLORA_BWD_REUSE_WT on another batch that shares workspace and W finds the copy."""
    import torch
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("wt", "bf16", 256, 320, [8, 24], [200, 300]), seed=2)
    lp = tlora.LayerProblem.from_numpy(p)
    dY = torch.from_numpy(p.dY).to(device="cuda", dtype=torch.bfloat16)
    Y, dX, dA, dB = lp.new_outputs()
    lp.fwd(Y); lp.bwd(dY, dX, dA, dB, reuse_S=True)
    dX.fill_(float("nan"))
    lp.fwd(Y); lp.bwd(dY, dX, dA, dB, reuse_S=True, flags=tlora.TLORA_BWD_REUSE_WT)
    torch.cuda.synchronize()
    _assert_ok(pu.compare(p, Y.float().cpu().numpy(), dX.float().cpu().numpy(), [a.cpu().numpy() for a in dA],
                          [b.cpu().numpy() for b in dB]), "reuse Wt")


def test_controller_in_the_loop():
    """Closed loop (Alg. 1, Phase 3): run a step with N nano-batches, feed a completion time to the controller, take
    its N for the next step.  The completion times that drive the controller are scripted (a fixed cost per
    nano-batch on top of a constant: what one GPU without communication to hide looks like), so the trajectory is
    the same on every machine; the steps themselves run on the GPU with each N the controller visits, and every one
    of them must stay correct.  Measured times are recorded but decide nothing."""
    import torch
    from oracle import aimd_oracle as aimd
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("loop", "bf16", 512, 512, [8, 16, 32, 64], [1024, 512, 2048, 512]), seed=9)
    lp = tlora.LayerProblem.from_numpy(p)
    dY = torch.from_numpy(p.dY).to(device="cuda", dtype=torch.bfloat16)
    Y, dX, dA, dB = lp.new_outputs()
    c = tlora.tlora_aimd_init(32, n_max=64)
    scripted = lambda n: 1.0 + 0.05 * n
    visited, measured = [], []
    for step in range(12):
        n = c.n
        visited.append(n)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        lp.fwd_nano(n, 64, Y)
        lp.bwd_nano(n, 64, dY, dX, dA, dB)
        torch.cuda.synchronize()
        measured.append(time.perf_counter() - t0)
        tlora.tlora_aimd_update(c, scripted(n))
        _assert_ok(pu.compare(p, Y.float().cpu().numpy(), dX.float().cpu().numpy(), [a.cpu().numpy() for a in dA],
                              [b.cpu().numpy() for b in dB]), f"controller loop, N = {n}")
    print("N visited:", visited, "measured ms:", [round(t * 1e3, 3) for t in measured])
    # the same scripted times through the oracle's controller give the same trajectory
    n_ref, ref, prev = 32, [], None
    for step in range(12):
        ref.append(n_ref)
        t = scripted(n_ref)
        n_ref, prev = aimd.aimd_update(n_ref, t, prev, n_max=64), t
    assert visited == ref and min(visited) < 32, (visited, ref)
