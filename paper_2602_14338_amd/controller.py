"""Host side of AERO's two-stage sampling (Sec. 4.1, Sec. 4.2 Strategy 1, App. C): decides how
many rollouts every query of a step receives.  Generation and verification are behind the
``draw(query, start, count) -> (rewards, lengths)`` callable of the caller (a simulator in the
tests); the groups that come out go to the curation call (aero_group_advantage), which applies
Strategies 2 and 3 to them.

  exploration   every query gets n_explore rollouts; c = number of correct ones
  rescue loop   queries with c <= S get n_extra more per iteration until an iteration brings a
                correct rollout; at most k_max iterations, at most n_max rollouts per query, and
                the whole step never generates more than n_budget * P rollouts
Readings of what the paper leaves open: rescue queries are served in query order inside an
iteration, the first increment that no longer fits the total budget ends the loop for every
query, and a query at its cap stops asking.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Tuple

import numpy as np


@dataclass
class Allocation:
    n: np.ndarray              # i32[P] rollouts generated per query
    c: np.ndarray              # i32[P] correct rollouts per query
    rescued_at: np.ndarray     # i32[P] 0: never in the rescue set, k >= 1: rescued in iteration k, -1: not rescued
    rewards: np.ndarray        # f32[R] ragged, generation order, query-major
    lengths: np.ndarray        # i32[R]
    group_offsets: np.ndarray  # i32[P+1]
    generated: int
    iterations: int


def allocate_rollouts(draw: Callable[[int, int, int], Tuple[np.ndarray, np.ndarray]], P: int, n_explore: int = 8,
                      n_extra: int = 2, k_max: int = 10, n_max: int = 32, n_budget: int = 16, S: int = 0) -> Allocation:
    if not (0 < n_explore <= n_max and n_extra > 0 and k_max >= 0 and 0 <= S <= n_explore // 2):
        raise ValueError("allocate_rollouts: inconsistent budgets")
    if n_explore > n_budget:
        raise ValueError("allocate_rollouts: the exploration pass alone exceeds the budget")
    cap_total = n_budget * P
    chunks_r = [[None] for _ in range(P)]     # per query: list of reward arrays in generation order
    chunks_l = [[None] for _ in range(P)]
    n = np.full(P, n_explore, np.int32)
    c = np.zeros(P, np.int32)
    for q in range(P):
        chunks_r[q][0], chunks_l[q][0] = draw(q, 0, n_explore)
        c[q] = int(np.count_nonzero(chunks_r[q][0] > 0))
    generated = int(n.sum())
    rescued_at = np.where(c <= S, -1, 0).astype(np.int32)
    pending = np.nonzero(c <= S)[0]
    iterations = 0
    while pending.size and iterations < k_max:
        iterations += 1
        pending = pending[n[pending] + n_extra <= n_max]            # capped queries drop out
        room = (cap_total - generated) // n_extra                   # increments that still fit
        served, unserved = pending[:max(room, 0)], pending[max(room, 0):]
        hit = np.zeros(served.size, bool)
        for j, q in enumerate(served):
            r, l = draw(int(q), int(n[q]), n_extra)
            chunks_r[q].append(r)
            chunks_l[q].append(l)
            k = int(np.count_nonzero(r > 0))
            c[q] += k
            hit[j] = k > 0
        n[served] += n_extra
        generated += n_extra * int(served.size)
        rescued_at[served[hit]] = iterations
        pending = np.concatenate([served[~hit], unserved])
        if unserved.size:                                            # the budget is exhausted
            break
    offsets = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    rewards = np.concatenate([np.asarray(a, np.float32) for q in range(P) for a in chunks_r[q]]) if P else np.zeros(0, np.float32)
    lengths = np.concatenate([np.asarray(a, np.int32) for q in range(P) for a in chunks_l[q]]) if P else np.zeros(0, np.int32)
    return Allocation(n=n, c=c, rescued_at=rescued_at, rewards=rewards, lengths=lengths, group_offsets=offsets,
                      generated=generated, iterations=iterations)
