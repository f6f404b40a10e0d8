"""Pins of the adaptive nano-batching oracle (Sec. 3.3) against things that do not come from it: trajectories
worked out by hand from the update rule, the halving count the paper states, and brute force over tokens."""
import math

import numpy as np
import pytest

from oracle import aimd_oracle as ao


def test_hand_worked_trajectory():
    # alpha = 4, beta = 1/2, tau = 2 % of the previous time.  By hand:
    #   first time 100: nothing to compare with                                -> 8
    #   90 <= 100 - 2     improved                                             -> 12
    #   89 <= 90 - 1.8 ?  89 > 88.2: not by the margin                         -> floor(12 / 2) = 6
    #   80 <= 89 - 1.78   improved                                             -> 10
    #   80 <= 80 - 1.6 ?  no                                                   -> 5
    #   81                no                                                   -> floor(2.5) = 2
    #   70                improved                                             -> 6
    assert ao.aimd_trace(8, [100, 90, 89, 80, 80, 81, 70]) == [8, 8, 12, 6, 10, 5, 2, 6]


def test_boundary_of_the_margin_counts_as_improvement():
    # T_t = T_{t-1} - tau exactly satisfies "<=" (values exactly representable: tau_rel = 1/4)
    assert ao.aimd_update(3, 75.0, 100.0, tau_rel=0.25) == 7
    assert ao.aimd_update(3, 75.0 + 2 ** -40, 100.0, tau_rel=0.25) == 1
    # tau = 0: an equal time still counts
    assert ao.aimd_update(3, 5.0, 5.0, tau_rel=0.0) == 7


@pytest.mark.parametrize("n0", [1, 2, 3, 7, 8, 64, 100, 1000])
def test_backoff_reaches_one_in_log2_steps(n0):
    # the paper: the way down from N to 1 takes O(log N) steps; with beta = 1/2 exactly floor(log2 N)
    trace = ao.aimd_trace(n0, [1.0] + [2.0 + i for i in range(40)])     # ever slower: always back off
    steps = next(i for i, n in enumerate(trace[1:]) if n == 1) if n0 > 1 else 0
    assert steps == (int(math.floor(math.log2(n0))) if n0 > 1 else 0)
    assert all(n == 1 for n in trace[1 + steps + 1:])                    # and stays at the floor of 1


def test_additive_increase_and_floor_and_limit():
    times = [100.0 * 0.9 ** i for i in range(6)]                         # 10 % faster every horizon
    assert ao.aimd_trace(1, times) == [1, 1, 5, 9, 13, 17, 21]
    assert ao.aimd_trace(1, times, alpha=3) == [1, 1, 4, 7, 10, 13, 16]
    assert ao.aimd_trace(1, times, n_max=10) == [1, 1, 5, 9, 10, 10, 10]
    assert ao.aimd_update(5, 2.0, 1.0) == 2 and ao.aimd_update(1, 2.0, 1.0) == 1     # floor(2.5), max(1, 0)
    assert ao.aimd_update(9, 2.0, 1.0, beta=0.75) == 6                               # floor(6.75)


@pytest.mark.parametrize("T,N,g", [(31744, 1, 512), (31744, 5, 512), (31744, 62, 512), (31744, 100, 512),
                                   (1000, 7, 1), (1000, 3, 64), (17, 4, 8), (0, 3, 16), (5, 1, 512)])
def test_partition_by_brute_force(T, N, g):
    b = ao.nano_bounds(T, N, g)
    assert len(b) == N + 1 and b[0] == 0 and b[-1] == T and all(x <= y for x, y in zip(b, b[1:]))
    # every token belongs to exactly one nano-batch, and boundaries fall on sample boundaries (or the end)
    owner = np.full(T, -1)
    for n in range(N):
        assert np.all(owner[b[n]:b[n + 1]] == -1)
        owner[b[n]:b[n + 1]] = n
    assert np.all(owner >= 0)
    assert all(x % g == 0 or x == T for x in b)
    # "approximately sum B_i / N samples each": sample counts differ by at most one
    units = [-(-(b[n + 1] - b[n]) // g) for n in range(N)]
    assert max(units) - min(units) <= 1


def test_sub_offsets_by_brute_force():
    offsets = [0, 300, 300, 1000, 1017, 2048]
    job_of = np.repeat(np.arange(5), np.diff(offsets))
    for N, g in [(1, 1), (3, 1), (4, 256), (7, 100), (40, 64)]:
        parts = ao.nano_split(offsets, N, g)
        total = np.zeros(5, dtype=int)
        for row0, row1, sub in parts:
            assert sub[0] == 0 and sub[-1] == row1 - row0 and all(x <= y for x, y in zip(sub, sub[1:]))
            counts = np.bincount(job_of[row0:row1], minlength=5)
            assert list(np.diff(sub)) == list(counts)                   # each job's rows inside the range
            # and they are the right rows: segment j of the nano-batch starts where job j's rows start
            for j in range(5):
                if counts[j]:
                    assert job_of[row0 + sub[j]] == j and job_of[row0 + sub[j + 1] - 1] == j
            total += counts
        assert list(total) == list(np.diff(offsets))
