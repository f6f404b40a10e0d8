"""CPU oracle of the adaptive nano-batching of Sec. 3.3.  TEST INFRASTRUCTURE ONLY.

Only the test-suite may import this module; the product path never does, and it shares no code with the
library.  Plain Python integers and floats, the steps in the paper's order and notation.

Controller (Sec. 3.3, "Adaptive Nano-Batching", the update rule printed as the second display equation):
    N_{t+1} = N_t + alpha                  if T_t <= T_{t-1} - tau
            = max(1, floor(beta * N_t))    otherwise
with alpha = 4 and beta = 1/2 by default.  The paper gives tau ("a stability margin to filter noise") no value:
here tau = tau_rel * T_{t-1} with tau_rel = 0.02.  The paper does not say what happens at the first horizon,
when there is no T_{t-1} to compare with: here the first observation is only recorded and N is kept.  An upper
limit n_max (0 = none) is this build's addition -- a batch cannot be cut into more nano-batches than it has
sequences -- and is applied after the rule.

Partition (same paragraph: the combined batch of the group is divided along the batch dimension into N
nano-batches of approximately sum_i B_i / N samples each, processed one after the other).  The batch is the
concatenation of the jobs' token segments; `granule` tokens (a sequence length) are the indivisible sample.
With U = ceil(T / granule) samples, nano-batch n covers samples floor(n U / N) .. floor((n + 1) U / N) - 1,
i.e. token rows [min(T, granule * floor(n U / N)), min(T, granule * floor((n + 1) U / N))).  Sizes differ by
at most one sample; a nano-batch is empty when N > U.  Inside a nano-batch, job j keeps the rows of its
segment that fall into the range.

Pinned by tests/test_aimd_pins.py: hand-computed trajectories, the halving count ceil(log2 N) the paper states
for the way down to 1, the boundary case T_t = T_{t-1} - tau, and partition invariants checked by brute force
over every token.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple


def aimd_update(n_t: int, t_now: float, t_prev: Optional[float], alpha: int = 4, beta: float = 0.5,
                tau_rel: float = 0.02, n_max: int = 0) -> int:
    """One application of the update rule.  `t_prev` is None at the first horizon."""
    if t_prev is None:
        n_next = n_t
    else:
        tau = tau_rel * t_prev
        if t_now <= t_prev - tau:
            n_next = n_t + alpha
        else:
            n_next = max(1, int(math.floor(beta * n_t)))
    if n_max > 0:
        n_next = min(n_next, n_max)
    return n_next


def aimd_trace(n0: int, times: Sequence[float], alpha: int = 4, beta: float = 0.5, tau_rel: float = 0.02,
               n_max: int = 0) -> List[int]:
    """N_0 and the N chosen after each observed completion time (len(times) + 1 entries)."""
    out = [n0]
    prev: Optional[float] = None
    n = n0
    for t in times:
        n = aimd_update(n, t, prev, alpha, beta, tau_rel, n_max)
        prev = t
        out.append(n)
    return out


def nano_bounds(total_tokens: int, n_nano: int, granule: int) -> List[int]:
    """Token boundaries b_0 = 0 <= b_1 <= ... <= b_N = T of the N nano-batches."""
    units = -(-total_tokens // granule)
    return [min(total_tokens, granule * ((n * units) // n_nano)) for n in range(n_nano + 1)]


def nano_sub_offsets(offsets: Sequence[int], b0: int, b1: int) -> List[int]:
    """Offsets (relative to b0) of the jobs' segments inside the row range [b0, b1)."""
    return [min(max(int(o), b0), b1) - b0 for o in offsets]


def nano_split(offsets: Sequence[int], n_nano: int, granule: int) -> List[Tuple[int, int, List[int]]]:
    """(row0, row1, sub-offsets) of every nano-batch."""
    bounds = nano_bounds(int(offsets[-1]), n_nano, granule)
    return [(bounds[n], bounds[n + 1], nano_sub_offsets(offsets, bounds[n], bounds[n + 1])) for n in range(n_nano)]
