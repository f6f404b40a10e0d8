"""GPU parity of the token-indexed entry points: tokens of the jobs interleaved in the batch, gathered by an index
and scattered back, against the token-by-token fp64 oracle."""
import numpy as np
import pytest

from oracle import indexed_oracle as io
from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


# dtype, d_in, d_out, path: "direct" = rows fetched through the index inside the kernels' loads (bf16 only),
# "gathered" = activations copied into job-sorted order first.  320 -> 264 has a contraction tail in the backward
# (264 = 8 * 32 + 8) and takes the generic shrink kernel there; 512 -> 768 runs the streaming kernels on both sides.
VARIANTS = [("bf16", 320, 264, "direct"), ("bf16", 320, 264, "gathered"), ("bf16", 512, 768, "direct"),
            ("f32", 96, 72, "gathered")]


@pytest.mark.parametrize("variant", VARIANTS, ids=["-".join(map(str, v)) for v in VARIANTS])
@pytest.mark.parametrize("shuffle", ["random", "interleaved_sequences", "identity"])
@pytest.mark.parametrize("reuse_S", [True, False])
def test_indexed_layer_matches_oracle(variant, shuffle, reuse_S):
    from paper_2602_07263_amd import tlora
    dtype, d_in, d_out, path = variant
    tlora.tlora_set_option("indexed_direct", 1 if path == "direct" else 0)
    try:
        _run_indexed(dtype, d_in, d_out, shuffle, reuse_S)
    finally:
        tlora.tlora_set_option("indexed_direct", 1)


def _run_indexed(dtype, d_in, d_out, shuffle, reuse_S):
    import torch
    from paper_2602_07263_amd import tlora
    ranks, tokens, scales = [8, 0, 24, 3, 64], [300, 40, 513, 70, 256], [2.0, 1.0, 0.5, 4.0, 2.0]
    print(f"indexed {dtype} {d_in}->{d_out} {shuffle} reuse_S={reuse_S}", flush=True)
    p = wk.generate(wk.custom("idx", dtype, d_in, d_out, ranks, tokens, scales), seed=13)
    T = int(p.offsets[-1])
    rng = np.random.default_rng(2)
    if shuffle == "random":
        idx = rng.permutation(T)
    elif shuffle == "identity":
        idx = np.arange(T)
    else:                                    # runs of 32 tokens ("sequences") of the jobs dealt round-robin
        job = np.repeat(np.arange(len(tokens)), tokens)
        key = np.concatenate([np.arange(t) // 32 for t in tokens])
        order = np.lexsort((job, key))       # batch order: by sequence number, then job
        idx = np.empty(T, dtype=np.int64)
        idx[order] = np.arange(T)            # idx[sorted position] = batch row
    idx = idx.astype(np.int32)
    inv = np.empty(T, dtype=np.int64); inv[idx] = np.arange(T)
    # the batch in its own order: row idx[i] of the batch is sorted row i
    X, dY = np.empty_like(p.X), np.empty_like(p.dY)
    X[idx], dY[idx] = p.X, p.dY
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=tdt).contiguous()
    lp = tlora.LayerProblem(dtype, d_in, d_out, ranks, p.offsets, scales, up(X), up(p.W), [up(a) for a in p.A],
                            [up(b) for b in p.B])
    ws_bytes = tlora.tlora_indexed_workspace_bytes(lp.prob)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    Y, dX, dA, dB = lp.new_outputs()
    Y.fill_(float("nan")); dX.fill_(float("nan"))
    for t in dA + dB:
        t.fill_(float("nan"))
    it = torch.from_numpy(idx).cuda()
    dYt = up(dY)
    st = int(torch.cuda.current_stream().cuda_stream)
    tlora.tlora_fwd_indexed(lp.prob, it.data_ptr(), Y.data_ptr(), ws.data_ptr(), ws_bytes, st)
    tlora.tlora_bwd_indexed(lp.prob, it.data_ptr(), dYt.data_ptr(), dX.data_ptr(),
                            [a.data_ptr() if a.numel() else 0 for a in dA], [b.data_ptr() if b.numel() else 0 for b in dB],
                            tlora.TLORA_BWD_REUSE_S if reuse_S else 0, ws.data_ptr(), ws_bytes, st)
    torch.cuda.synchronize()
    Yr, dXr, dAr, dBr = io.forward_backward(X, p.W, p.A, p.B, scales, p.offsets, idx, dY)
    tol = pu.BF16_TOL if dtype == "bf16" else pu.F32_TOL
    res = {"Y": pu.worst_ratio(Y.float().cpu().numpy(), Yr, tol), "dX": pu.worst_ratio(dX.float().cpu().numpy(), dXr, tol),
           "dA": max([pu.worst_ratio(a.cpu().numpy(), r, tol) for a, r in zip(dA, dAr)] + [0.0]),
           "dB": max([pu.worst_ratio(b.cpu().numpy(), r, tol) for b, r in zip(dB, dBr)] + [0.0])}
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"{dtype}/{shuffle}: worst error / tolerance ratios {res}"


@pytest.mark.parametrize("variant", [VARIANTS[0], VARIANTS[1], VARIANTS[3]], ids=["bf16-direct", "bf16-gathered", "f32"])
def test_row_list_entries_out_of_range_are_forced_into_the_batch(variant):
    """The list is the caller's device data and cannot be checked on the host; the library works on a copy with every
    entry forced into [0, T), so a bad list gives wrong rows, never an access outside the tensors.  Checked here: a list
    with entries below 0 and at or beyond T behaves exactly like the list with those entries replaced by 0 / T - 1 --
    the gradient sums in full, Y and dX on every row that the forced list names once."""
    import torch
    from paper_2602_07263_amd import tlora
    dtype, d_in, d_out, path = variant
    ranks, tokens, scales = [8, 0, 24, 3, 64], [300, 40, 513, 70, 256], [2.0, 1.0, 0.5, 4.0, 2.0]
    print(f"indexed, list out of range, {dtype} {d_in}->{d_out} {path}", flush=True)
    p = wk.generate(wk.custom("idx_bad", dtype, d_in, d_out, ranks, tokens, scales), seed=14)
    T = int(p.offsets[-1])
    rng = np.random.default_rng(3)
    idx = rng.permutation(T).astype(np.int64)
    bad_at = rng.choice(T, size=9, replace=False)
    idx[bad_at] = [-1, -7, -2**31, T, T + 1, T + 4096, 2**30, 2**31 - 1, -T]
    forced = np.clip(idx, 0, T - 1)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    up = lambda a: torch.from_numpy(a).to(device="cuda", dtype=tdt).contiguous()
    lp = tlora.LayerProblem(dtype, d_in, d_out, ranks, p.offsets, scales, up(p.X), up(p.W), [up(a) for a in p.A],
                            [up(b) for b in p.B])
    ws_bytes = tlora.tlora_indexed_workspace_bytes(lp.prob)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    Y, dX, dA, dB = lp.new_outputs()
    it = torch.from_numpy(idx.astype(np.int32)).cuda()
    dYt = up(p.dY)
    st = int(torch.cuda.current_stream().cuda_stream)
    tlora.tlora_set_option("indexed_direct", 1 if path == "direct" else 0)
    try:
        tlora.tlora_fwd_indexed(lp.prob, it.data_ptr(), Y.data_ptr(), ws.data_ptr(), ws_bytes, st)
        tlora.tlora_bwd_indexed(lp.prob, it.data_ptr(), dYt.data_ptr(), dX.data_ptr(),
                                [a.data_ptr() if a.numel() else 0 for a in dA],
                                [b.data_ptr() if b.numel() else 0 for b in dB], 0, ws.data_ptr(), ws_bytes, st)
        torch.cuda.synchronize()
    finally:
        tlora.tlora_set_option("indexed_direct", 1)
    Yr, dXr, dAr, dBr = io.forward_backward(p.X, p.W, p.A, p.B, scales, p.offsets, forced, p.dY)
    once = np.flatnonzero(np.bincount(forced, minlength=T) == 1)
    assert once.size >= T - 20
    tol = pu.BF16_TOL if dtype == "bf16" else pu.F32_TOL
    res = {"Y": pu.worst_ratio(Y.float().cpu().numpy()[once], Yr[once], tol),
           "dX": pu.worst_ratio(dX.float().cpu().numpy()[once], dXr[once], tol),
           "dA": max([pu.worst_ratio(a.cpu().numpy(), r, tol) for a, r in zip(dA, dAr)] + [0.0]),
           "dB": max([pu.worst_ratio(b.cpu().numpy(), r, tol) for b, r in zip(dB, dBr)] + [0.0])}
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"{dtype}/{path}: worst error / tolerance ratios {res}"
