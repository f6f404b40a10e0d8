"""tlora_fwd_noalloc (the forward for callers that cannot allocate: its intermediates live in a device array that
is part of the library) against tlora_fwd on a caller-provided workspace: same kernels, so Y must agree bit for
bit -- on two calls in a row, the second on a smaller problem (the array keeps the first call's contents), in
both dtypes; the result is also held to the oracle's tolerance.  A problem beyond the array's size is refused
before anything is launched.  Last: the call recorded into a captured stream (what the entry point exists for) and
replayed three times, with eager calls on another problem through the same array in between."""
import numpy as np
import pytest

from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu

# name, d_in, d_out, ranks, tokens, scales: several 256-row tiles with ragged tails, then a smaller problem
FIRST = ("noalloc_first", 512, 768, [3, 16, 40, 0, 130], [300, 700, 129, 40, 260], [2.0, 0.5, 1.0, 2.0, 1.5])
SECOND = ("noalloc_second", 256, 384, [8, 5], [70, 33], [2.0, 3.0])


def _both_ways(case, dtype, seed):
    import torch
    from paper_2602_07263_amd import tlora
    from oracle import tlora_oracle as orc
    name, d_in, d_out, ranks, tokens, scales = case
    p = wk.generate(wk.custom(name, dtype, d_in, d_out, ranks, tokens, scales), seed=seed)
    lp = tlora.LayerProblem.from_numpy(p)
    Y_ws, _, _, _ = lp.new_outputs()
    Y_na = torch.empty_like(Y_ws)
    Y_ws.fill_(float("nan"))
    Y_na.fill_(float("nan"))
    print(f"tlora_fwd / tlora_fwd_noalloc {name} {dtype} seed {seed}", flush=True)
    lp.fwd(Y_ws)
    tlora.tlora_fwd_noalloc(lp.prob, Y_na.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()
    a, b = Y_ws.float().cpu().numpy(), Y_na.float().cpu().numpy()
    assert np.all(np.isfinite(b)), f"{name}/{dtype}: unwritten or non-finite outputs"
    assert np.array_equal(a, b), f"{name}/{dtype}: differs from tlora_fwd in {np.count_nonzero(a != b)} elements"
    ref, _ = orc.forward(p.X, p.W, p.A, p.B, p.scales, p.offsets)
    tol = pu.BF16_TOL if dtype == "bf16" else pu.F32_TOL
    assert pu.worst_ratio(b, ref, tol) <= 1.0
    return lp


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_two_calls_in_a_row_second_smaller(dtype):
    _both_ways(FIRST, dtype, seed=21)
    _both_ways(SECOND, dtype, seed=22)
    _both_ways(FIRST, dtype, seed=23)      # and back up: stale contents of the smaller call in between


def test_problem_beyond_the_scratch_is_refused():
    import torch
    from paper_2602_07263_amd import tlora
    # 16384 tokens at rank 256 into 4096 -> 4096: the packed adapters alone exceed the 16 MiB array
    import ctypes
    T, d, r = 16384, 4096, 256
    X = torch.zeros(T, d, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(d, d, dtype=torch.bfloat16, device="cuda")
    A = [torch.zeros(d, r, dtype=torch.bfloat16, device="cuda")]
    B = [torch.zeros(r, d, dtype=torch.bfloat16, device="cuda")]
    lp = tlora.LayerProblem("bf16", d, d, [r], [0, T], [2.0], X, W, A, B)
    Y = torch.full((T, d), 7.0, dtype=torch.bfloat16, device="cuda")
    rc = tlora.lib().tlora_fwd_noalloc(ctypes.byref(lp.prob), ctypes.c_void_p(Y.data_ptr()), None)
    assert rc == tlora.TLORA_ESCRATCH
    assert "scratch" in tlora.tlora_strerror(rc)
    torch.cuda.synchronize()
    assert bool((Y == 7.0).all()), "a refused call must not launch anything"


def test_noalloc_forward_replays_from_a_captured_stream():
    import torch
    from paper_2602_07263_amd import tlora
    mk = lambda case, seed: tlora.LayerProblem.from_numpy(wk.generate(wk.custom(case[0], "bf16", *case[1:]), seed=seed))
    lp, other = mk(FIRST, 31), mk(SECOND, 32)
    Y_ref, _, _, _ = lp.new_outputs()
    Y_other, _, _, _ = other.new_outputs()
    lp.fwd(Y_ref)
    Y = torch.empty_like(Y_ref)
    st = lambda: int(torch.cuda.current_stream().cuda_stream)
    print("noalloc: set-up call before the capture", flush=True)
    tlora.tlora_fwd_noalloc(lp.prob, Y.data_ptr(), st())
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_ref)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    print("noalloc: capture", flush=True)
    with torch.cuda.graph(graph, stream=side):
        tlora.tlora_fwd_noalloc(lp.prob, Y.data_ptr(), st())
    for rep in range(3):
        Y.fill_(float("nan"))
        # eager work between the replays: another problem through the same scratch array
        tlora.tlora_fwd_noalloc(other.prob, Y_other.data_ptr(), st())
        torch.cuda.synchronize()
        print(f"noalloc: replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_ref), f"replay {rep}: {int((Y != Y_ref).sum())} elements differ from the eager call"
