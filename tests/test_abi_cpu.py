"""Host-side checks that need no GPU: the C-ABI library loads and exports what include/tlora.h
declares, rejects bad arguments before touching the device, and its integer bookkeeping (padded
ranks, row tiles with their first / last job) is bit-identical to the oracle's independently written
version; the private layout of the intermediates is checked for validity, not against the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import tlora_oracle as orc
from paper_2602_07263_amd import tlora, workloads as wk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _problem(ranks, tokens, d_in=64, d_out=128, dtype=tlora.TLORA_BF16, X=0x1000, W=0x2000):
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    J = len(ranks)
    return tlora.make_problem(dtype, d_in, d_out, ranks, off, [2.0] * J, X, W, [0x3000] * J, [0x4000] * J)


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "tlora.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = set(re.findall(r"\b(tlora_[a-z_]+)\s*\(", text))
    assert declared == set(tlora.EXPORTS)
    L = tlora.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert tlora.tlora_version().startswith("tlora-gfx950")
    assert tlora.tlora_strerror(0) == "ok" and "workspace" in tlora.tlora_strerror(-4)


def test_invalid_problems_are_rejected_on_the_host():
    L = tlora.lib()
    ws = ctypes.c_void_p(0x10000)

    def fwd(prob, Y=0x5000, ws_ptr=ws, nbytes=1 << 40):
        return L.tlora_fwd(ctypes.byref(prob), ctypes.c_void_p(Y), ws_ptr, ctypes.c_size_t(nbytes), None)

    ok, _k0 = _problem([4, 8], [10, 20])
    assert tlora.tlora_workspace_bytes(ok) > 0
    bad_dtype, _k1 = _problem([4], [10], dtype=7)
    assert fwd(bad_dtype) == -3 and tlora.tlora_workspace_bytes(bad_dtype) == 0
    bad_d, _k2 = _problem([4], [10], d_in=60)
    assert fwd(bad_d) == -1
    neg_rank, _k3 = _problem([-1], [10])
    assert fwd(neg_rank) == -1
    big_rank, _k4 = _problem([4096], [10])
    assert fwd(big_rank) == -1
    decreasing, keep = _problem([4, 4], [10, 5])
    keep[1][2] = 3          # offsets = [0, 10, 3]
    assert fwd(decreasing) == -1
    nonzero_start, keep2 = _problem([4], [10])
    keep2[1][0] = 1
    assert fwd(nonzero_start) == -1
    null_x, _k5 = _problem([4], [10], X=0)
    assert fwd(null_x) == -2
    assert fwd(ok, Y=0x5000, ws_ptr=None) == -4            # no workspace
    assert fwd(ok, nbytes=16) == -4                       # workspace too small
    assert fwd(ok, ws_ptr=ctypes.c_void_p(0x10010)) == -4  # workspace not 256-byte aligned
    misaligned, _k6 = _problem([4], [10], X=0x1008)
    assert fwd(misaligned) == -7
    assert L.tlora_fwd(None, None, None, 0, None) == -2
    # backward: dA and dB must be given together; unknown flags are refused
    dA = (ctypes.c_void_p * 2)(0x6000, 0x7000)
    rc = L.tlora_bwd(ctypes.byref(ok), ctypes.c_void_p(0x5000), None, dA, None, 0, ws, ctypes.c_size_t(1 << 40), None)
    assert rc == -2
    with pytest.raises(tlora.TloraError):
        tlora.tlora_set_option("no_such_option", 1)
    with pytest.raises(tlora.TloraError):
        tlora.tlora_set_option("shrink_rows", 100)


def _check_packed_layout(prob, plan, ranks, off):
    """Where job j's block of the intermediates lies in the workspace is the library's own choice (the paper fixes
    no layout), so it is not compared with the oracle: it only has to be a valid layout -- blocks in job order that
    do not overlap, each with room for the job's T_j x rpad_j elements, starting on 16-byte boundaries (two-byte
    elements), and all of it inside the workspace the library asks for."""
    soff = plan["soff"]
    assert soff[0] == 0 and len(soff) == len(ranks) + 1
    for j, r in enumerate(ranks):
        need = (int(off[j + 1]) - int(off[j])) * orc.padded_rank(r)
        assert soff[j + 1] - soff[j] >= need, f"job {j}: block too small"
        assert (soff[j] * 2) % 16 == 0
    assert 4 * 2 * soff[-1] <= tlora.tlora_workspace_bytes(prob)      # S and dS, hi and lo planes


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_plan_bookkeeping_is_bit_exact(cfg):
    wl = wk.config(cfg)
    off = wl.offsets
    for proj in wl.projections[:2]:
        prob, _keep = tlora.make_problem(tlora.TLORA_BF16, proj.d_in, proj.d_out, wl.ranks, off, wl.scales,
                                         0x1000, 0x2000, [0x3000] * wl.num_jobs, [0x4000] * wl.num_jobs)
        plan = tlora.tlora_plan_dump(prob)
        assert plan["rpad"] == [orc.padded_rank(r) for r in wl.ranks]
        assert plan["tiles"] == orc.row_tiles(off, plan["tile_rows"])
        _check_packed_layout(prob, plan, wl.ranks, off)


def test_plan_handles_empty_segments_and_rank_zero():
    ranks, tokens = [3, 0, 9, 1], [0, 300, 0, 5]
    prob, _keep = _problem(ranks, tokens)
    off = np.concatenate([[0], np.cumsum(tokens)])
    plan = tlora.tlora_plan_dump(prob)
    assert plan["rpad"] == [8, 0, 16, 8]
    _check_packed_layout(prob, plan, ranks, off)
    assert plan["tiles"] == orc.row_tiles(off, plan["tile_rows"])
    # all-empty batch: no tiles
    prob0, _k = _problem([4, 4], [0, 0])
    assert tlora.tlora_plan_dump(prob0)["tiles"] == []


def test_workspace_grows_with_rank_work_not_with_dense_weights():
    # Sec. 3.3: no per-job d_in x d_out buffer.  The workspace holds ONE bf16 d_in x d_out matrix for all jobs
    # together (the transposed copy of the frozen W that the backward runs against); everything else is
    # rank-sized.  Doubling d_in and d_out (4x the dense weight) with few tokens must grow that remainder far
    # less than 4x.
    small, _a = _problem([8] * 8, [16] * 8, d_in=1024, d_out=1024)
    large, _b = _problem([8] * 8, [16] * 8, d_in=2048, d_out=2048)
    rest_s = tlora.tlora_workspace_bytes(small) - 1024 * 1024 * 2
    rest_l = tlora.tlora_workspace_bytes(large) - 2048 * 2048 * 2
    assert 0 < rest_l < 2048 * 2048 * 2        # less than one more dense bf16 matrix, for all 8 jobs together
    assert rest_l < 2.6 * rest_s               # ~linear in (d_in + d_out)
    one, _e = _problem([64], [128], d_in=2048, d_out=2048)     # the same rank total and tokens in a single job
    assert abs(tlora.tlora_workspace_bytes(large) - tlora.tlora_workspace_bytes(one)) < 0.25 * 2048 * 2048 * 2
    # and it is linear in sum_j T_j r_j
    a, _c = _problem([16] * 4, [1000] * 4)
    b, _d = _problem([16] * 4, [2000] * 4)
    assert tlora.tlora_workspace_bytes(b) < 2.1 * tlora.tlora_workspace_bytes(a)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 and as C++ with no other includes."""
    import os
    import subprocess
    import tempfile
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hdr = os.path.join(root, "include", "tlora.h")
    with tempfile.TemporaryDirectory() as td:
        for name, cc, std in (("t.c", "gcc", "-std=c99"), ("t.cpp", "g++", "-std=c++11")):
            src = os.path.join(td, name)
            with open(src, "w") as f:
                f.write('#include "%s"\nint main(void) { tlora_problem_t p; (void)p; return sizeof(tlora_aimd_t) > 0 ? 0 : 1; }\n' % hdr)
            r = subprocess.run([cc, std, "-Wall", "-Werror", "-pedantic", "-fsyntax-only", src], capture_output=True, text=True)
            assert r.returncode == 0, r.stderr


def _attn_struct(ranks, tokens, seq, d_model=256, n_heads=4, n_kv=2, head_dim=128, dtype=tlora.TLORA_BF16):
    J = len(ranks)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    keep = [(ctypes.c_int32 * J)(*ranks), (ctypes.c_int64 * (J + 1))(*[int(o) for o in off]), (ctypes.c_float * J)(*[1.0] * J),
            (ctypes.c_int64 * len(seq))(*seq), (ctypes.c_void_p * J)(*[0x3000] * J)]
    p = tlora.tlora_attn_t(dtype, J, d_model, n_heads, n_kv, head_dim, 10000.0, 1e-5, keep[0], keep[1], keep[2],
                           len(seq) - 1, keep[3], 0x1000, 0x2000, 0x5000, 0x6000, 0x7000, 0x8000, *([keep[4]] * 8))
    return p, keep


def test_attention_arguments_are_checked_on_the_host():
    """Workspace sizing and argument validation of the attention entry points touch no device."""
    L = tlora.lib()
    seq = (ctypes.c_int64 * 3)(0, 100, 300)
    small = L.tlora_attention_workspace_bytes(2, seq, 4)
    assert small > 0 and small % 256 == 0
    # grows with tokens x heads (the fp32 row statistics of the backward) and with the longest sequence (rotary table)
    seq2 = (ctypes.c_int64 * 3)(0, 1000, 3000)
    assert L.tlora_attention_workspace_bytes(2, seq2, 4) > small
    assert L.tlora_attention_workspace_bytes(2, seq, 0) == 0                      # no heads
    assert L.tlora_attention_workspace_bytes(2, (ctypes.c_int64 * 3)(0, 300, 100), 4) == 0   # offsets go down
    assert L.tlora_attention_workspace_bytes(2, (ctypes.c_int64 * 3)(1, 100, 300), 4) == 0   # do not start at 0
    ws = ctypes.c_void_p(0x10000)
    args = lambda hq, hkv, hd: (ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000), ctypes.c_void_p(0x3000), ctypes.c_void_p(0x4000),
                                ctypes.c_void_p(0x5000), 2, seq, hq, hkv, hd, ws, ctypes.c_size_t(1 << 40), None)
    assert L.tlora_attention_fwd(*args(4, 2, 64)) == tlora.TLORA_EINVAL            # head size
    assert L.tlora_attention_fwd(*args(3, 2, 128)) == tlora.TLORA_EINVAL           # heads not a multiple
    a = list(args(4, 2, 128)); a[11] = ctypes.c_size_t(16)
    assert L.tlora_attention_fwd(*a) == tlora.TLORA_EWORKSPACE
    a = list(args(4, 2, 128)); a[0] = None
    assert L.tlora_attention_fwd(*a) == tlora.TLORA_ENULL
    a = list(args(4, 2, 128)); a[1] = ctypes.c_void_p(0x2008)
    assert L.tlora_attention_fwd(*a) == tlora.TLORA_EALIGN
    assert L.tlora_rope(ctypes.c_void_p(0x1000), 2, seq, 4, 128, ctypes.c_float(0.5), 0, ws, ctypes.c_size_t(1 << 40), None) \
        == tlora.TLORA_EINVAL                                                       # rotary base must exceed 1


def test_block_and_layer_structs_are_checked_on_the_host():
    L = tlora.lib()
    p, keep = _attn_struct([8, 4], [96, 64], [0, 96, 160])
    need = L.tlora_attn_workspace_bytes(ctypes.byref(p))
    assert need > 0
    bad, _k = _attn_struct([8, 4], [96, 64], [0, 96, 150])                          # sequences cover 150 of 160 tokens
    assert L.tlora_attn_workspace_bytes(ctypes.byref(bad)) == 0
    bad, _k = _attn_struct([8, 4], [96, 64], [0, 96, 160], dtype=tlora.TLORA_F32)    # bf16 only
    assert L.tlora_attn_workspace_bytes(ctypes.byref(bad)) == 0
    bad, _k = _attn_struct([8, 4], [96, 64], [0, 96, 160], n_heads=4, n_kv=3)
    assert L.tlora_attn_workspace_bytes(ctypes.byref(bad)) == 0
    assert L.tlora_attn_fwd(ctypes.byref(p), ctypes.c_void_p(0x9000), ctypes.c_void_p(0x10000), ctypes.c_size_t(need - 1), None) \
        == tlora.TLORA_EWORKSPACE
    # a layer needs both halves on the same jobs
    J = 2
    mlp = tlora.tlora_mlp_t(tlora.TLORA_BF16, J, 256, 512, keep[0], keep[1], keep[2], None, 0x2000, 1e-5, 0x5000, 0x6000, 0x7000,
                            *([keep[4]] * 6))
    layer = tlora.tlora_layer_t(p, mlp)
    total = L.tlora_layer_workspace_bytes(ctypes.byref(layer))
    assert total > need
    other = (ctypes.c_int32 * J)(8, 16)                                              # ranks differ between the halves
    mlp2 = tlora.tlora_mlp_t(tlora.TLORA_BF16, J, 256, 512, other, keep[1], keep[2], None, 0x2000, 1e-5, 0x5000, 0x6000, 0x7000,
                             *([keep[4]] * 6))
    assert L.tlora_layer_workspace_bytes(ctypes.byref(tlora.tlora_layer_t(p, mlp2))) == 0
    mlp3 = tlora.tlora_mlp_t(tlora.TLORA_BF16, J, 128, 512, keep[0], keep[1], keep[2], None, 0x2000, 1e-5, 0x5000, 0x6000, 0x7000,
                             *([keep[4]] * 6))                                       # d_model differs
    assert L.tlora_layer_workspace_bytes(ctypes.byref(tlora.tlora_layer_t(p, mlp3))) == 0


def test_plan_cache_returns_the_same_plan_as_a_fresh_build():
    """Plans are cached by the contents of (dtype, sizes, ranks, offsets) and the tiling options: the cached plan, the
    plan after 200 other problems have pushed it out, and the plan with the cache switched off must be identical, and
    a tiling option that changes the plan must not be answered from an entry built under another value."""
    rng = np.random.default_rng(5)
    ref_prob, _k = _problem([8, 40, 3, 130], [300, 129, 260, 513], d_in=256, d_out=384)
    first = tlora.tlora_plan_dump(ref_prob)
    ws_first = tlora.tlora_workspace_bytes(ref_prob)
    assert tlora.tlora_plan_dump(ref_prob) == first                      # served from the cache
    for _ in range(200):                                                  # more distinct problems than the cache holds
        J = int(rng.integers(1, 6))
        q, _kq = _problem([int(r) for r in rng.integers(0, 70, J)], [int(t) for t in rng.integers(0, 600, J)])
        tlora.tlora_plan_dump(q)
    assert tlora.tlora_plan_dump(ref_prob) == first and tlora.tlora_workspace_bytes(ref_prob) == ws_first
    try:
        tlora.tlora_set_option("plan_cache", 0)
        assert tlora.tlora_plan_dump(ref_prob) == first and tlora.tlora_workspace_bytes(ref_prob) == ws_first
        tlora.tlora_set_option("plan_cache", 1)
        tlora.tlora_set_option("grad_tokens", 64)                         # shorter dA / dB chunks: more partial tiles
        ws_small_chunks = tlora.tlora_workspace_bytes(ref_prob)
        tlora.tlora_set_option("grad_tokens", 256)
        assert tlora.tlora_workspace_bytes(ref_prob) == ws_first
        assert ws_small_chunks >= ws_first
    finally:
        tlora.tlora_set_option("plan_cache", 1)
        tlora.tlora_set_option("grad_tokens", 256)


def _random_plan_problem(rng):
    """Problem shapes of the kinds the workloads have: even and skewed token counts, empty segments, rank 0, ranks up
    to the maximum, feature sizes that are and are not multiples of 64."""
    J = int(rng.integers(1, 41))
    kind = int(rng.integers(0, 4))
    if kind == 0:
        tokens = rng.integers(0, 700, J)
    elif kind == 1:                                                   # heavy tail, many tiny or empty jobs
        tokens = (rng.pareto(0.8, J) * 20).astype(np.int64) % 20000
    elif kind == 2:
        tokens = rng.choice([0, 1, 31, 32, 33, 255, 256, 257, 4095, 4096, 4097], J)
    else:
        tokens = rng.integers(0, 3, J)                                # nearly empty batch (sometimes T = 0)
    rank_set = [0, 1, 3, 8, 16, 33, 64, 96, 127, 128, 129, 256, 384, 513, 1024]
    ranks = [int(rng.choice(rank_set)) if rng.random() < 0.8 else int(rng.integers(0, 1025)) for _ in range(J)]
    d_in = int(rng.choice([8, 64, 72, 256, 1000, 4096]))
    d_out = int(rng.choice([8, 64, 136, 512, 1024, 12288]))
    dtype = tlora.TLORA_BF16 if rng.random() < 0.85 else tlora.TLORA_F32
    return _problem(ranks, [int(t) for t in tokens], d_in=d_in, d_out=d_out, dtype=dtype)


def test_planner_self_check_on_random_problems():
    """Every table entry and workspace region the kernels index is verified on the host, for 1500 random problems under
    every tiling option (unit heights of the shrink, token chunks of the dA / dB reduction), forward-only and full."""
    rng = np.random.default_rng(20240607)
    settings = [(0, 256), (32, 64), (64, 1024), (128, 4096), (0, 64)]
    try:
        for i in range(1500):
            rows, chunk = settings[i % len(settings)]
            tlora.tlora_set_option("shrink_rows", rows)
            tlora.tlora_set_option("grad_tokens", chunk)
            prob, _keep = _random_plan_problem(rng)
            for fwd_only in (False, True):
                rc, bad = tlora.tlora_plan_check(prob, fwd_only)
                assert (rc, bad) == (0, 0), (i, fwd_only, rows, chunk, bad, list(prob.ranks[:prob.num_jobs]),
                                             list(prob.offsets[:prob.num_jobs + 1]), prob.d_in, prob.d_out, prob.dtype)
    finally:
        tlora.tlora_set_option("shrink_rows", 0)
        tlora.tlora_set_option("grad_tokens", 256)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_planner_self_check_on_the_five_configurations(cfg):
    wl = wk.config(cfg)
    for proj in wl.projections:
        prob, _keep = tlora.make_problem(tlora.TLORA_F32 if wl.dtype == "f32" else tlora.TLORA_BF16, proj.d_in, proj.d_out,
                                         wl.ranks, wl.offsets, wl.scales, 0x1000, 0x2000, [0x3000] * wl.num_jobs,
                                         [0x4000] * wl.num_jobs)
        for fwd_only in (False, True):
            assert tlora.tlora_plan_check(prob, fwd_only) == (0, 0)


def test_planner_self_check_reports_the_problem_s_own_errors():
    prob, _keep = _problem([8, 8], [10, 10], d_in=60)                  # d_in not a multiple of 8
    rc, bad = tlora.tlora_plan_check(prob)
    assert rc == tlora.TLORA_EINVAL and bad == 0


def test_sizes_beyond_the_stated_limits_are_refused_on_the_host():
    """No pointer is touched: the fake addresses of _problem are never dereferenced by the planner."""
    L = tlora.lib()

    def ws(ranks, tokens, **kw):
        prob, _keep = _problem(ranks, tokens, **kw)
        return tlora.tlora_workspace_bytes(prob), tlora.tlora_plan_check(prob)[0]
    at_limit = ws([8], [4096], d_in=1 << 20, d_out=64)
    assert at_limit[0] > 0 and at_limit[1] == 0                                             # at the limit: fine
    assert ws([8], [4096], d_in=(1 << 20) + 8, d_out=64) == (0, tlora.TLORA_EINVAL)
    assert ws([8], [4096], d_in=64, d_out=(1 << 20) + 8) == (0, tlora.TLORA_EINVAL)
    assert ws([8], [(1 << 24) + 1], d_in=64, d_out=64) == (0, tlora.TLORA_EINVAL)
    assert ws([8], [1 << 24], d_in=64, d_out=64)[1] == 0                                    # 65536 x 1 tiles
    assert ws([8], [1 << 24], d_in=64, d_out=1 << 15) == (0, tlora.TLORA_EINVAL)            # 65536 x 128 tiles > 2^22
    assert ws([8], [1 << 20], d_in=64, d_out=1 << 18)[1] == 0                               # 4096 x 1024 tiles = 2^22
    assert ws([1025], [10]) == (0, tlora.TLORA_EINVAL)
    J = 8192                                                                                # padded ranks sum to 2^23
    prob, _keep = tlora.make_problem(tlora.TLORA_BF16, 64, 64, [1024] * J, list(range(J + 1)), [1.0] * J, 0x1000, 0x2000,
                                     [0x3000] * J, [0x4000] * J)
    assert tlora.tlora_workspace_bytes(prob) == 0 and tlora.tlora_plan_check(prob)[0] == tlora.TLORA_EINVAL
    J = 32769
    prob, _keep = tlora.make_problem(tlora.TLORA_BF16, 64, 64, [1] * J, list(range(J + 1)), [1.0] * J, 0x1000, 0x2000,
                                     [0x3000] * J, [0x4000] * J)
    assert tlora.tlora_workspace_bytes(prob) == 0 and tlora.tlora_plan_check(prob)[0] == tlora.TLORA_EINVAL
