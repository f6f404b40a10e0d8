"""The native scheduler (host code of the C-ABI library; no device involved) against the oracle: groups, traces and
times must agree bit for bit on random queues over a measured-looking step-time model."""
import ctypes

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2602_07263_amd import tlora

MODEL = dict(tokens=[256.0, 1024.0, 4096.0, 16384.0, 32768.0], ms=[0.31, 0.42, 1.13, 3.94, 7.7], rho=2.5e-7, kappa=0.013)


def _jobs(rng, n):
    return [dict(tokens=int(rng.choice([512, 1024, 2048, 4096]) * rng.choice([1, 2, 4, 8]) // 4 + int(rng.integers(0, 3)) * 64),
                 rank=int(rng.choice([2, 4, 8, 16])), steps=int(rng.integers(3, 80)),
                 urgency=float(rng.choice([1.0, 1.0, 1.3, 2.0])), max_slowdown=float(rng.choice([1.5, 3.0, 1e300])))
            for _ in range(n)]


@pytest.mark.parametrize("seed", range(12))
def test_partition_and_step_time_match_oracle(seed):
    rng = np.random.default_rng(seed)
    jobs = _jobs(rng, int(rng.integers(1, 14)))
    s = tlora.Scheduler(MODEL, jobs)
    groups = s.partition()
    assert groups == so.partition(MODEL, jobs)
    for g in groups:
        assert s.step_ms(g) == so.step_ms(MODEL, jobs, g)          # bit for bit


@pytest.mark.parametrize("seed", range(6))
def test_simulation_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    jobs = _jobs(rng, int(rng.integers(2, 10)))
    horizon = int(rng.choice([4, 16, 50]))
    trace, jct, now = tlora.Scheduler(MODEL, jobs).simulate(horizon)
    t_r, jct_r, now_r = so.simulate(MODEL, jobs, horizon)
    assert trace == [(g, n) for g, n in t_r]
    assert jct == jct_r and now == now_r


def test_native_simulation_reproduces_the_hand_worked_trace():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "sched_three_job_trace.json")) as f:
        g = json.load(f)
    trace, jct, now = tlora.Scheduler(g["model"], g["jobs"]).simulate(g["horizon"])
    assert [[grp, n] for grp, n in trace] == g["trace"]
    assert np.allclose(jct, g["jct_ms"], rtol=1e-12, atol=0.0) and abs(now - g["makespan_ms"]) <= 1e-12 * now


def test_scheduler_rejects_bad_arguments():
    L = tlora.lib()
    s = tlora.Scheduler(MODEL, [dict(tokens=100, rank=4)])
    out = ctypes.c_double()
    m = (ctypes.c_int32 * 1)(5)
    assert L.tlora_sched_step_ms(ctypes.byref(s.model), 1, s.jobs, m, 1, ctypes.byref(out)) != 0      # member out of range
    bad = tlora.Scheduler(dict(tokens=[10.0, 10.0], ms=[1.0, 2.0], rho=0.0), [dict(tokens=100, rank=4)])
    with pytest.raises(tlora.TloraError):
        bad.partition()                                                                                # tokens not ascending
    with pytest.raises(tlora.TloraError):
        tlora.Scheduler(MODEL, [dict(tokens=0, rank=4)]).partition()
    with pytest.raises(tlora.TloraError):
        tlora.Scheduler(MODEL, [dict(tokens=10, rank=4, max_slowdown=0.5)]).partition()
    assert tlora.Scheduler(MODEL, []).partition() == []
