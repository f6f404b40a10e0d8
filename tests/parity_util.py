"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI and compare it with
the fp64 oracle element by element (all rows, or a row sample for Y / dX on large problems)."""
from __future__ import annotations

import numpy as np

from oracle import tlora_oracle as orc

BF16_TOL = 2e-2     # |err| <= 2e-2 * (1 + |ref|): bf16 inputs, fp32 accumulation
F32_TOL = 1e-5      # |err| <= 1e-5 * (1 + |ref|) and ||err||_F <= 1e-5 ||ref||_F for the fp32 configuration


def worst_ratio(got: np.ndarray, ref: np.ndarray, tol: float) -> float:
    if ref.size == 0:
        return 0.0
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    return float(np.max(np.abs(got - ref) / (tol * (1.0 + np.abs(ref)))))


def frob_rel(got, ref) -> float:
    n = float(np.linalg.norm(ref))
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref)) / n if n > 0 else 0.0


def sample_rows(offsets, tile_rows: int, rng: np.random.Generator, per_job: int = 64) -> np.ndarray:
    """Rows that always include segment edges, tile edges, whole short segments and random rows."""
    T = int(offsets[-1])
    rows = set()
    for j in range(len(offsets) - 1):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        if hi <= lo:
            continue
        if hi - lo <= 64:
            rows.update(range(lo, hi))
        else:
            rows.update([lo, lo + 1, hi - 2, hi - 1])
            rows.update(int(r) for r in rng.integers(lo, hi, per_job))
    for edge in range(tile_rows, T, tile_rows):
        rows.update([edge - 1, edge])
    if T:
        rows.update([0, T - 1])
    return np.array(sorted(r for r in rows if 0 <= r < T), dtype=np.int64)


def run_gpu(p, reuse_S: bool = True, want_dX: bool = True, want_grads: bool = True):
    """Upload, run fwd + bwd through the C ABI, download.  Returns numpy arrays (float32/float64-able)."""
    import torch
    from paper_2602_07263_amd import tlora
    lp = tlora.LayerProblem.from_numpy(p)
    tdt = torch.bfloat16 if p.dtype == "bf16" else torch.float32
    dY = torch.from_numpy(p.dY).to(device="cuda", dtype=tdt)
    Y, dX, dA, dB = lp.new_outputs()
    # poison the outputs so unwritten elements are caught
    Y.fill_(float("nan")); dX.fill_(float("nan"))
    for t in dA + dB:
        t.fill_(float("nan"))
    lp.fwd(Y)
    lp.bwd(dY, dX if want_dX else None, dA if want_grads else None, dB if want_grads else None, reuse_S=reuse_S)
    torch.cuda.synchronize()
    return (Y.float().cpu().numpy(), dX.float().cpu().numpy(), [a.cpu().numpy() for a in dA],
            [b.cpu().numpy() for b in dB], lp)


def compare(p, Y, dX, dA, dB, rows=None, tol=None):
    """Worst error ratios (<= 1 passes) of each output against the oracle."""
    tol = tol if tol is not None else (BF16_TOL if p.dtype == "bf16" else F32_TOL)
    off = p.offsets
    Yr, _ = orc.forward(p.X, p.W, p.A, p.B, p.scales, off, rows=rows)
    dXr, dAr, dBr, _ = orc.backward(p.X, p.W, p.A, p.B, p.scales, off, p.dY, rows=rows)
    sel = slice(None) if rows is None else rows
    out = {"Y": worst_ratio(Y[sel], Yr, tol), "dX": worst_ratio(dX[sel], dXr, tol)}
    out["dA"] = max([worst_ratio(a, r, tol) for a, r in zip(dA, dAr)] + [0.0])
    out["dB"] = max([worst_ratio(b, r, tol) for b, r in zip(dB, dBr)] + [0.0])
    if p.dtype == "f32":
        out["frob"] = max([frob_rel(Y[sel], Yr), frob_rel(dX[sel], dXr)] +
                          [frob_rel(a, r) for a, r in zip(dA, dAr)] + [frob_rel(b, r) for b, r in zip(dB, dBr)]) / tol
    return out


def rms_floor_ratio(got, ref, tol: float) -> float:
    """Worst |err| / (tol (m + |ref|)) with m = max(1, rms(ref)): for gradients that are long token sums of products
    of tensors a block stores in bf16 between its kernels, one-ulp flips of those reach a sum as noise relative to
    the sum's typical size (its rms), also on entries that happen to be near zero."""
    if ref.size == 0:
        return 0.0
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), "non-finite values in GPU output"
    m = max(1.0, float(np.sqrt(np.mean(ref * ref))))
    return float(np.max(np.abs(got - ref) / (tol * (m + np.abs(ref)))))


def bf16_store(a):
    """Storage hook of the block oracles: round a float64 tensor to bf16 (RNE) and widen it again."""
    from paper_2602_07263_amd import workloads as wk
    return wk.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def block_report(label, Out, dX, grads, oracle, tol: float, stored_hook, rms_floor_on_acts: bool = False):
    """Compare a block's GPU results (torch tensors) with its fp64 oracle twice: against the plain oracle, which
    rounds nothing (the definition in float64), and against the oracle that rounds the tensors the block keeps in
    memory (`stored_hook`), which shows the share of the error that the storage points explain.  Both are printed
    and both must hold the tolerance: the returned ratios are the element-wise worse of the two.
    `oracle(store)` returns (Out, dX, {name: (dA list, dB list)})."""
    got_out, got_dX = Out.float().cpu().numpy(), dX.float().cpu().numpy()
    got_g = {n: ([a.cpu().numpy() for a in grads[n][0]], [b.cpu().numpy() for b in grads[n][1]]) for n in grads}
    act = rms_floor_ratio if rms_floor_on_acts else worst_ratio
    out = {}
    for kind, hook in (("rounding oracle", stored_hook), ("plain oracle", lambda a: a)):
        out_r, dX_r, g_r = oracle(hook)
        res = {"Out": act(got_out, out_r, tol), "dX": act(got_dX, dX_r, tol)}
        for n in got_g:
            res["dA_" + n] = max([rms_floor_ratio(a, r, tol) for a, r in zip(got_g[n][0], g_r[n][0])] + [0.0])
            res["dB_" + n] = max([rms_floor_ratio(b, r, tol) for b, r in zip(got_g[n][1], g_r[n][1])] + [0.0])
        print(f"{label} vs {kind}: worst error / tolerance", {k: round(v, 3) for k, v in res.items()}, flush=True)
        out[kind] = res
    return {k: max(out["rounding oracle"][k], out["plain oracle"][k]) for k in out["plain oracle"]}
