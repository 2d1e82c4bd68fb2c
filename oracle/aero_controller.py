"""Plain-loop checker for the rollout-allocation loop of AERO's two stages.

TEST INFRASTRUCTURE ONLY (same rules as aero_oracle.py: nothing in the product imports it and
it shares no code with the product's controller).

What it follows: Sec. 4.1 (every query first gets n_explore rollouts; the success count c of
that pass stratifies the queries), Sec. 4.2 Strategy 1 (queries with c <= S enter the rescue
loop: n_extra more rollouts per iteration until an iteration brings at least one correct
rollout or the budget is gone) and App. C "Iterative Rejection Sampling" / "Budget
Constraints" (at most K_max iterations, increment Delta n, per-query cap n_max, total cap
n_budget * |P| including the exploration pass).  Readings: inside an iteration the rescue
queries are served in query order, and the first increment that does not fit the total budget
ends the loop for everybody; a query that reached n_max simply stops receiving rollouts.
Queries outside the rescue set receive nothing beyond the exploration pass (their
allocation stays n_p, or shrinks by rejection sampling, which the curation step does).
"""
import numpy as np


def allocate(sim, P, n_explore=8, n_extra=2, k_max=10, n_max=32, n_budget=16, S=0):
    """Returns per query: n (rollouts generated), c (correct ones), rescued_at (iteration, 1-based,
    at which the first success arrived; 0 = was never in the rescue set; -1 = never rescued),
    the ragged rewards / lengths in generation order and the total number generated."""
    total_cap = n_budget * P
    n = [0] * P
    c = [0] * P
    rewards = [[] for _ in range(P)]
    lengths = [[] for _ in range(P)]
    generated = 0
    for q in range(P):
        r, l = sim.draw(q, 0, n_explore)
        rewards[q].extend(float(x) for x in r)
        lengths[q].extend(int(x) for x in l)
        n[q] = n_explore
        c[q] = int(sum(1 for x in r if x > 0))
        generated += n_explore
    rescued_at = [0] * P
    waiting = [q for q in range(P) if c[q] <= S]
    for q in waiting:
        rescued_at[q] = -1
    out_of_budget = False
    it = 0
    while waiting and it < k_max and not out_of_budget:
        it += 1
        nxt = []
        for q in waiting:
            if out_of_budget:
                nxt.append(q)
                continue
            if n[q] + n_extra > n_max:
                continue                      # capped: stays unrescued, asks for nothing more
            if generated + n_extra > total_cap:
                out_of_budget = True
                nxt.append(q)
                continue
            r, l = sim.draw(q, n[q], n_extra)
            rewards[q].extend(float(x) for x in r)
            lengths[q].extend(int(x) for x in l)
            n[q] += n_extra
            generated += n_extra
            hits = int(sum(1 for x in r if x > 0))
            c[q] += hits
            if hits > 0:
                rescued_at[q] = it
            else:
                nxt.append(q)
        waiting = nxt
    offsets = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    return dict(n=np.array(n, np.int32), c=np.array(c, np.int32), rescued_at=np.array(rescued_at, np.int32),
                rewards=np.array([x for r in rewards for x in r], np.float32),
                lengths=np.array([x for l in lengths for x in l], np.int32),
                group_offsets=offsets, generated=generated, iterations=it)
