"""Host-side checks of the adaptive nano-batching entry points (no GPU): the library's controller and partition
against the oracle, bit for bit, and their error paths."""
import numpy as np
import pytest

from oracle import aimd_oracle as ao
from paper_2602_07263_amd import tlora, workloads as wk


def _prob(ranks, tokens, d_in=64, d_out=128, dtype=tlora.TLORA_BF16):
    J = len(ranks)
    off = np.concatenate([[0], np.cumsum(tokens)]).astype(np.int64)
    return tlora.make_problem(dtype, d_in, d_out, ranks, off, [2.0] * J, 0x100000, 0x200000, [0x3000] * J, [0x4000] * J), off


@pytest.mark.parametrize("seed", range(6))
def test_controller_matches_oracle_on_random_time_series(seed):
    rng = np.random.default_rng(seed)
    alpha = int(rng.integers(1, 9)); beta = float(rng.choice([0.5, 0.25, 0.75, 0.9])); tau = float(rng.choice([0.0, 0.02, 0.1]))
    n_max = int(rng.choice([0, 7, 40])); n0 = int(rng.integers(1, 30))
    times = list(np.abs(rng.normal(10.0, 1.0, 200)) * np.exp(-0.002 * np.arange(200)))
    c = tlora.tlora_aimd_init(n0, alpha, beta, tau, n_max)
    got = [c.n] + [tlora.tlora_aimd_update(c, t) for t in times]
    want = ao.aimd_trace(min(n0, n_max) if n_max else n0, times, alpha, beta, tau, n_max)
    assert got == want
    assert min(got) >= 1 and (n_max == 0 or max(got) <= n_max)


def test_controller_scripted_cases():
    c = tlora.tlora_aimd_init(8)                         # defaults of the paper: alpha 4, beta 1/2
    assert [tlora.tlora_aimd_update(c, t) for t in [100, 90, 89, 80, 80, 81, 70]] == [8, 12, 6, 10, 5, 2, 6]
    c = tlora.tlora_aimd_init(64)
    down = [tlora.tlora_aimd_update(c, 1.0 + i) for i in range(9)]
    assert down == [64, 32, 16, 8, 4, 2, 1, 1, 1]        # log2(64) halvings, then the floor of 1
    assert c.n == 1 and c.have_prev == 1


def test_controller_rejects_bad_parameters():
    L = tlora.lib()
    c = tlora.tlora_aimd_t()
    import ctypes
    bad = [(0, 4, 0.5, 0.02, 0), (1, 0, 0.5, 0.02, 0), (1, 4, 0.0, 0.02, 0), (1, 4, 1.0, 0.02, 0),
           (1, 4, 0.5, -0.1, 0), (1, 4, 0.5, 0.02, -1), (1, 4, float("nan"), 0.02, 0)]
    for args in bad:
        assert L.tlora_aimd_init(ctypes.byref(c), *args) == -1
    assert L.tlora_aimd_init(None, 1, 4, 0.5, 0.02, 0) == -2
    assert L.tlora_aimd_init(ctypes.byref(c), 3, 4, 0.5, 0.02, 0) == 0
    assert L.tlora_aimd_update(ctypes.byref(c), -1.0, None) == -1
    assert L.tlora_aimd_update(ctypes.byref(c), float("nan"), None) == -1
    assert L.tlora_aimd_update(None, 1.0, None) == -2


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_partition_matches_oracle_on_the_workload_configs(cfg):
    wl = wk.config(cfg)
    (prob, _keep), off = _prob(wl.ranks, wl.tokens)
    for N, g in [(1, 512), (2, 512), (7, 2048), (16, 1), (61, 333)]:
        want = ao.nano_split(list(off), N, g)
        for n in range(N):
            assert tlora.tlora_nano_split(prob, N, g, n) == want[n]


def test_partition_edge_cases_and_errors():
    (prob, _k), off = _prob([4, 8, 0, 3], [300, 0, 17, 700])
    for N, g in [(1, 1), (3, 64), (40, 64), (2000, 1)]:
        want = ao.nano_split(list(off), N, g)
        assert [tlora.tlora_nano_split(prob, N, g, n) for n in range(N)] == want
    (empty, _k2), _ = _prob([4], [0])
    assert tlora.tlora_nano_split(empty, 3, 16, 2) == (0, 0, [0, 0])
    L = tlora.lib()
    import ctypes
    for N, g, n in [(0, 1, 0), (3, 0, 0), (3, 1, 3), (3, 1, -1)]:
        assert L.tlora_nano_split(ctypes.byref(prob), N, g, n, None, None, None) == -1
    assert tlora.tlora_nano_workspace_bytes(prob, 0, 1) == 0
    # a nano-batch never needs more workspace than the whole batch, and the need shrinks as N grows
    full = tlora.tlora_workspace_bytes(prob)
    w = [tlora.tlora_nano_workspace_bytes(prob, N, 1) for N in (1, 2, 8)]
    assert w[0] == full and w[0] >= w[1] >= w[2] > 0
