"""CPU oracle of the adapter scheduler's grouping phase (Sec. 3.4, Algorithm 1 Phase 1) on one device, over a
measured step-time model.  TEST INFRASTRUCTURE ONLY.

Algorithm 1 keeps a queue of jobs (and already merged groups), sorted by urgency (descending) and residual resources
(ascending).  It pops the first entry as the seed, looks for the partner whose union with the seed has the highest
joint throughput, merges and re-inserts if there is a beneficial one, and finalizes the seed otherwise.  The paper
leaves Throughput(.), the residual, the urgency and "beneficial" to the implementation; this build fixes them so:

    step_ms(G)    = curve(sum_j tokens_j) + rho * sum_j tokens_j * rank_j + kappa * (|G| - 1)
                    curve = piecewise-linear interpolation of measured (tokens, ms) points, flat below the first
                    point, continued along the last segment above the last point; kappa = measured cost of one
                    more job in a fused call (packing its adapters, its ragged tile edges)
    throughput(G) = sum_j tokens_j / step_ms(G)                                   (tokens per ms)
    residual(G)   = 1 - throughput(G) / peak,   peak = max_i tokens_i / ms_i       (idle share of the device)
    urgency(G)    = max of the members' urgencies
    slowdown of j in G = step_ms(G) / step_ms({j})  must stay <= max_slowdown_j       (Sec. 3.4's constraint)
    a merge of seed and k is beneficial when throughput(seed + k) exceeds what time-sharing the device between
    the two gives: (tokens_seed + tokens_k) / (step_ms(seed) + step_ms(k))

Ties: sort by (-urgency, residual, smallest job id); among equally good partners the first in queue order wins.
Everything is IEEE double arithmetic in exactly the order written here.

The outer loop of Algorithm 1 on one device (`simulate`): group, run the group for up to `horizon` steps, update
the members' progress, recompute urgencies (slowdown so far: elapsed time over the standalone time of the steps
done, at least one step), repeat until every job has finished.

Pinned by tests/test_sched_pins.py (hand-worked example, exhaustive search on small queues, invariants).
"""
from __future__ import annotations


def curve(model, tokens):
    xs, ys = model["tokens"], model["ms"]
    t = float(tokens)
    if t <= xs[0]:
        return float(ys[0])
    i = len(xs) - 2
    for k in range(len(xs) - 1):
        if t < xs[k + 1]:
            i = k
            break
    return ys[i] + (ys[i + 1] - ys[i]) * ((t - xs[i]) / (xs[i + 1] - xs[i]))


def step_ms(model, jobs, members):
    total = 0
    work = 0.0
    for j in members:
        total += jobs[j]["tokens"]
        work += float(jobs[j]["tokens"]) * float(jobs[j]["rank"])
    return curve(model, total) + model["rho"] * work + model.get("kappa", 0.0) * float(len(members) - 1)


def tokens_of(jobs, members):
    return sum(jobs[j]["tokens"] for j in members)


def throughput(model, jobs, members):
    return float(tokens_of(jobs, members)) / step_ms(model, jobs, members)


def peak(model):
    best = 0.0
    for x, y in zip(model["tokens"], model["ms"]):
        best = max(best, float(x) / y)
    return best


def residual(model, jobs, members):
    return 1.0 - throughput(model, jobs, members) / peak(model)


def feasible(model, jobs, members):
    t = step_ms(model, jobs, members)
    return all(t / step_ms(model, jobs, [j]) <= jobs[j]["max_slowdown"] for j in members)


def _key(model, jobs, urgency, members):
    return (-max(urgency[j] for j in members), residual(model, jobs, members), min(members))


def next_group(model, jobs, active, urgency):
    """One pass of Algorithm 1's Phase 1 over the queue `active` (job indices): the finalized group, as a sorted
    list of job indices.  `urgency[j]` is the current urgency of job j."""
    items = [[j] for j in active]
    while True:
        items.sort(key=lambda m: _key(model, jobs, urgency, m))
        seed, rest = items[0], items[1:]
        best, best_thr = None, 0.0
        for k, other in enumerate(rest):
            union = sorted(seed + other)
            if not feasible(model, jobs, union):
                continue
            thr = throughput(model, jobs, union)
            shared = float(tokens_of(jobs, union)) / (step_ms(model, jobs, seed) + step_ms(model, jobs, other))
            if not thr > shared:
                continue
            if best is None or thr > best_thr:
                best, best_thr = k, thr
        if best is None:
            return sorted(seed)
        merged = sorted(seed + rest[best])
        items = [m for k, m in enumerate(rest) if k != best] + [merged]


def partition(model, jobs, urgency=None):
    """Groups for all jobs: Phase 1 repeated on what is left (the groups a cluster would run side by side)."""
    urgency = list(urgency) if urgency is not None else [jb.get("urgency", 1.0) for jb in jobs]
    active = list(range(len(jobs)))
    groups = []
    while active:
        g = next_group(model, jobs, active, urgency)
        groups.append(g)
        active = [j for j in active if j not in g]
    return groups


def simulate(model, jobs, horizon):
    """Algorithm 1's outer loop on one device.  jobs[j]['steps'] = training steps to run.  Returns (trace, jct, now):
    trace = [(group, steps run)], jct[j] = completion time of job j in ms."""
    n = len(jobs)
    left = [jb["steps"] for jb in jobs]
    done = [0] * n
    alone = [step_ms(model, jobs, [j]) for j in range(n)]
    jct = [0.0] * n
    now = 0.0
    trace = []
    active = [j for j in range(n) if left[j] > 0]
    while active:
        urgency = [1.0] * n
        for j in active:
            if now > 0.0:
                urgency[j] = now / (alone[j] * float(max(done[j], 1)))
        g = next_group(model, jobs, active, urgency)
        steps = min(horizon, min(left[j] for j in g))
        now = now + float(steps) * step_ms(model, jobs, g)
        for j in g:
            left[j] -= steps
            done[j] += steps
            if left[j] == 0:
                jct[j] = now
        trace.append((g, steps))
        active = [j for j in active if left[j] > 0]
    return trace, jct, now
