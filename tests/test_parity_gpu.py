"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded
inputs.  Tolerances: bf16 |err| <= 2e-2 (1 + |ref|); fp32 |err| <= 1e-5 (1 + |ref|) and a 1e-5
Frobenius bound.  Small problems are compared element by element; the full-size configurations on
all of dA_j / dB_j and on a row sample of Y / dX that holds every segment and tile edge."""
import numpy as np
import pytest

from paper_2602_07263_amd import workloads as wk
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _assert_ok(res, label):
    bad = {k: v for k, v in res.items() if not v <= 1.0}
    assert not bad, f"{label}: worst error / tolerance ratios {res}"


def test_cfg0_fp32_full():
    p = wk.generate(wk.config(0))
    Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=True)
    _assert_ok(pu.compare(p, Y, dX, dA, dB), "cfg0")
    Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=False)
    _assert_ok(pu.compare(p, Y, dX, dA, dB), "cfg0 recompute S")


RAGGED = [
    # name, d_in, d_out, ranks, tokens, scales
    ("ragged_small", 192, 320, [1, 3, 8, 20, 0, 64, 96], [1, 17, 0, 333, 70, 300, 513], [0.5, 4.0, 2.0, 1.0, 2.0, 3.0, 0.75]),
    ("one_token", 64, 64, [1], [1], [2.0]),
    ("tile_edges", 256, 512, [8, 16, 24], [256, 255, 257], [2.0, 2.0, 2.0]),
    ("rank_256_straddle", 320, 264, [256, 3, 130], [100, 700, 90], [1.5, 2.0, 0.5]),
    ("narrow_features", 8, 8, [2, 5], [40, 300], [2.0, 1.0]),
    # the largest legal rank (TLORA_MAX_RANK = 1024: eight rank blocks per shrink / dA-dB unit column) next to a rank
    # that ends inside a block; feature sizes that take the streaming kernels, then sizes that take the generic ones
    ("rank_max_streaming", 256, 320, [1024, 513], [300, 129], [1.0, 2.0]),
    ("rank_max_generic", 136, 200, [1024, 8, 513], [70, 33, 260], [0.5, 2.0, 1.5]),
]


@pytest.mark.parametrize("case", RAGGED, ids=[c[0] for c in RAGGED])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_ragged_edge_cases_full(case, dtype):
    name, d_in, d_out, ranks, tokens, scales = case
    p = wk.generate(wk.custom(name, dtype, d_in, d_out, ranks, tokens, scales), seed=11)
    for reuse in (True, False):
        Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=reuse)
        _assert_ok(pu.compare(p, Y, dX, dA, dB), f"{name}/{dtype}/reuse={reuse}")


def test_all_segments_empty_and_rank_zero_jobs():
    p = wk.generate(wk.custom("rank0", "bf16", 64, 128, [0, 0], [5, 300]), seed=3)
    Y, dX, dA, dB, _ = pu.run_gpu(p)
    _assert_ok(pu.compare(p, Y, dX, dA, dB), "rank0")
    p = wk.generate(wk.custom("empty", "bf16", 64, 128, [4, 9], [0, 0]), seed=3)
    Y, dX, dA, dB, _ = pu.run_gpu(p)
    assert all(np.all(a == 0) for a in dA) and all(np.all(b == 0) for b in dB)


def test_cfg1_bf16_full():
    p = wk.generate(wk.config(1))
    Y, dX, dA, dB, _ = pu.run_gpu(p)
    _assert_ok(pu.compare(p, Y, dX, dA, dB), "cfg1")


def test_zero_B_gives_backbone_only_and_jobs_do_not_leak():
    wl = wk.custom("leak", "bf16", 128, 256, [8, 16, 4], [100, 300, 50])
    p = wk.generate(wl, seed=5)
    Y, dX, dA, dB, _ = pu.run_gpu(p)
    # perturb job 1 only: outputs of jobs 0 and 2 must be bit-identical
    p2 = wk.generate(wl, seed=5)
    lo, hi = int(p.offsets[1]), int(p.offsets[2])
    p2.X[lo:hi] = wk.round_to_bf16(p2.X[lo:hi] * 2 + 1)
    p2.A[1] = wk.round_to_bf16(p2.A[1] * 3)
    p2.B[1] = wk.round_to_bf16(p2.B[1] - 1)
    Y2, dX2, dA2, dB2, _ = pu.run_gpu(p2)
    for j in (0, 2):
        sl = slice(int(p.offsets[j]), int(p.offsets[j + 1]))
        assert np.array_equal(Y[sl], Y2[sl]) and np.array_equal(dX[sl], dX2[sl])
        assert np.array_equal(dA[j], dA2[j]) and np.array_equal(dB[j], dB2[j])
    # B = 0: dA = 0 exactly
    p3 = wk.generate(wl, seed=5)
    p3.B = [np.zeros_like(b) for b in p3.B]
    Y3, dX3, dA3, dB3, _ = pu.run_gpu(p3)
    assert all(np.all(a == 0) for a in dA3)
    _assert_ok(pu.compare(p3, Y3, dX3, dA3, dB3), "B=0")


def test_cached_plan_takes_scales_and_pointers_from_every_call():
    """Two problems with the same sizes, ranks and offsets share one cached plan; their scales, activations and
    adapters differ (other tensors at other addresses): each must match its own oracle, with the cache on and off."""
    from paper_2602_07263_amd import tlora
    shape = ("bf16", 256, 384, [8, 40, 3], [300, 129, 260])
    a = wk.generate(wk.custom("cache_a", *shape, [2.0, 0.5, 1.0]), seed=31)
    b = wk.generate(wk.custom("cache_b", *shape, [0.25, 3.0, 4.0]), seed=32)
    try:
        for cache in (1, 0, 1):
            tlora.tlora_set_option("plan_cache", cache)
            for p in (a, b, a):
                Y, dX, dA, dB, _ = pu.run_gpu(p)
                _assert_ok(pu.compare(p, Y, dX, dA, dB), f"{p.name if hasattr(p, 'name') else 'problem'} cache={cache}")
    finally:
        tlora.tlora_set_option("plan_cache", 1)


def test_run_to_run_determinism():
    p = wk.generate(wk.custom("det", "bf16", 512, 768, [8, 64, 33], [700, 1300, 129]), seed=2)
    a = pu.run_gpu(p)
    b = pu.run_gpu(p)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for x, y in zip(a[2] + a[3], b[2] + b[3]):
        assert np.array_equal(x, y)


# every (configuration, projection) pair of the three large bf16 workloads, at full size, in the launch configuration
# the benchmark times (default options, backward reusing the forward's S): cfg2's gate / up / down, cfg3's q / k / v / o /
# gate / up / down, cfg4's up / down.  dA_j / dB_j are compared in full; Y / dX on every segment edge, every tile
# edge, whole short segments and 256 random rows per job.
FULL_SIZE = [(2, 0), (2, 1), (2, 2), (3, 0), (3, 1), (3, 2), (3, 3), (3, 4), (3, 5), (3, 6), (4, 0), (4, 1)]


@pytest.mark.parametrize("cfg,proj", FULL_SIZE, ids=[f"cfg{c}-{wk.config(c).projections[q].name}" for c, q in FULL_SIZE])
def test_full_size_configs_sampled(cfg, proj):
    wl = wk.config(cfg)
    print(f"full size cfg{cfg} projection {wl.projections[proj].name}", flush=True)
    p = wk.generate(wl, proj)
    Y, dX, dA, dB, lp = pu.run_gpu(p)
    rows = pu.sample_rows(p.offsets, 256, np.random.default_rng(cfg * 10 + proj), per_job=256)
    _assert_ok(pu.compare(p, Y, dX, dA, dB, rows=rows), f"cfg{cfg}/{wl.projections[proj].name}")


DEFAULT_OPTIONS = {"dx_transposed_w": 1, "shrink_rows": 0, "shrink_stages": 4, "grad_tokens": 256}
TILINGS = [
    {"dx_transposed_w": 0},
    {"shrink_rows": 64, "shrink_stages": 8},
    {"grad_tokens": 64},
    {"grad_tokens": 2048, "shrink_rows": 64},
    {"shrink_rows": 32},
    {"shrink_rows": 128},
    {"shrink_rows": 128, "shrink_stages": 8},
]


@pytest.mark.parametrize("opts", TILINGS, ids=["-".join(f"{k}{v}" for k, v in o.items()) for o in TILINGS])
def test_results_do_not_depend_on_the_tiling(opts):
    """Nano-batch shapes (workgroup layout of the GEMM, token rows per shrink unit, token chunk of the dA / dB
    reduction) change the summation order only: every tiling must meet the oracle tolerance (Sec. 3.3: the
    nano-batch size is a performance knob, not part of the result)."""
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("tiling", "bf16", 384, 640, [1, 12, 256, 40, 130], [300, 17, 700, 1, 520],
                              [0.5, 2.0, 1.0, 4.0, 2.0]), seed=21)
    try:
        for k, v in opts.items():
            tlora.tlora_set_option(k, v)
        Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=False)
        _assert_ok(pu.compare(p, Y, dX, dA, dB), f"tiling {opts}")
    finally:
        for k, v in DEFAULT_OPTIONS.items():
            tlora.tlora_set_option(k, v)


@pytest.mark.parametrize("opts", [{"shrink_rows": 128}, {"shrink_rows": 128, "shrink_stages": 8}, {"shrink_rows": 64}],
                         ids=["rows128", "rows128-stages8", "rows64"])
def test_streaming_shrink_with_k_steps_of_32(opts):
    """Contraction lengths that are multiples of 32 but not of 64 (96 forward, 160 backward) take the streaming
    shrink's 32-wide K-steps, also in its 128-row, eight-wave form."""
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("k32", "bf16", 96, 160, [3, 40, 130, 8], [300, 129, 260, 513], [2.0, 0.5, 1.0, 3.0]), seed=41)
    try:
        for k, v in opts.items():
            tlora.tlora_set_option(k, v)
        Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=False)
        _assert_ok(pu.compare(p, Y, dX, dA, dB), f"K-steps of 32, {opts}")
    finally:
        for k, v in DEFAULT_OPTIONS.items():
            tlora.tlora_set_option(k, v)


def test_kernel_timing_hooks_count_every_launch():
    from paper_2602_07263_amd import tlora
    p = wk.generate(wk.custom("prof", "bf16", 128, 256, [8, 16], [100, 200]), seed=4)
    tlora.tlora_profile(True)
    try:
        pu.run_gpu(p, reuse_S=True)
        prof = tlora.tlora_profile_read()
    finally:
        tlora.tlora_profile(False)
    assert prof["gemm_fwd"][1] == 1 and prof["gemm_bwd"][1] == 1
    assert prof["shrink"][1] == 2 and prof["rank_grad"][1] == 2 and prof["grad_reduce"][1] == 2
    assert prof["pack"][1] == 2 and prof["f32"][1] == 0 and prof["w_transpose"][1] == 1
    assert all(ms >= 0.0 for ms, _ in prof.values()) and prof["gemm_fwd"][0] > 0.0


def _random_case(rng):
    """A small random problem that stresses the tile logic: short and long contractions (fewer K-steps than the
    pipeline is deep, a K tail, adapters only), widths off the 256 grid, ranks from 0 to beyond one 32-step, many
    jobs per row tile and jobs spanning several tiles."""
    d_in = int(rng.choice([8, 24, 32, 40, 64, 96, 200, 256, 328, 512, 776]))
    d_out = int(rng.choice([8, 16, 72, 256, 264, 520]))
    J = int(rng.integers(1, 9))
    ranks = [int(rng.choice([0, 1, 2, 5, 8, 16, 31, 32, 33, 64, 100, 130, 256, 300])) for _ in range(J)]
    tokens = [int(rng.choice([0, 1, 3, 31, 32, 33, 100, 255, 256, 257, 400, 700])) for _ in range(J)]
    scales = [float(rng.choice([0.5, 1.0, 2.0, 4.0])) for _ in range(J)]
    return d_in, d_out, ranks, tokens, scales


@pytest.mark.parametrize("seed", range(24))
def test_random_small_problems(seed):
    rng = np.random.default_rng(1000 + seed)
    d_in, d_out, ranks, tokens, scales = _random_case(rng)
    p = wk.generate(wk.custom(f"rand{seed}", "bf16", d_in, d_out, ranks, tokens, scales), seed=seed)
    Y, dX, dA, dB, _ = pu.run_gpu(p, reuse_S=bool(seed & 1))
    _assert_ok(pu.compare(p, Y, dX, dA, dB), f"seed {seed}: d {d_in}->{d_out} ranks {ranks} tokens {tokens}")
