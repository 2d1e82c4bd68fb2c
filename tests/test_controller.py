"""Rollout-allocation loop (Sec. 4.1, Strategy 1, App. C budget constraints), CPU only: the
plain-loop checker against what the paper fixes, then the product's controller against it."""
import numpy as np
import pytest

import aero_inputs as ai
from oracle import aero_controller as ctl_ref
from oracle import aero_oracle as orc
from paper_2602_14338_amd.controller import allocate_rollouts


def test_simulator_positions_are_fixed():
    sim = ai.RolloutSimulator(3, P=5)
    r_all, l_all = sim.draw(2, 0, 32)
    r_mid, l_mid = sim.draw(2, 10, 4)
    assert np.array_equal(r_all[10:14], r_mid) and np.array_equal(l_all[10:14], l_mid)
    assert set(np.unique(r_all)) <= {0.0, 1.0} and l_all.min() >= 128 and l_all.max() <= 2048
    with pytest.raises(ValueError):
        sim.draw(0, 30, 4)


def test_checker_deterministic_corner_cases():
    P = 6
    # never correct: 2 more per iteration for K_max = 10 iterations -> 8 + 20 = 28 <= n_max
    sim = ai.RolloutSimulator(0, P, p_q=np.zeros(P))
    out = ctl_ref.allocate(sim, P, n_budget=32)
    assert (out["n"] == 28).all() and (out["c"] == 0).all() and (out["rescued_at"] == -1).all()
    assert out["iterations"] == 10 and out["generated"] == 28 * P
    # the per-query cap binds before K_max
    out = ctl_ref.allocate(sim, P, n_budget=32, n_max=14)
    assert (out["n"] == 14).all() and out["iterations"] == 4      # 3 increments fit, the 4th finds everybody capped
    # always correct: nobody is in the rescue set, nothing beyond the exploration pass
    sim1 = ai.RolloutSimulator(0, P, p_q=np.ones(P))
    out = ctl_ref.allocate(sim1, P)
    assert (out["n"] == 8).all() and (out["rescued_at"] == 0).all() and out["iterations"] == 0
    assert out["generated"] == 8 * P == out["rewards"].size == out["lengths"].size
    # total budget n_budget * P = 16 P: the exploration pass takes 8 P, so 4 P increments of 2 fit:
    # iteration 1..4 serve all P queries, iteration 5 finds the budget gone
    out = ctl_ref.allocate(sim, P, n_budget=16)
    assert out["generated"] == 16 * P and (out["n"] == 16).all() and out["iterations"] == 5
    # an odd budget: queries are served in order until the next increment does not fit
    out = ctl_ref.allocate(sim, P, n_budget=9)                      # 6 rollouts left = 3 increments
    assert out["n"].tolist() == [10, 10, 10, 8, 8, 8] and out["generated"] == 54 and out["iterations"] == 1


@pytest.mark.parametrize("seed", range(5))
def test_checker_invariants_and_group_of_two_on_first_success(seed):
    P = 40
    sim = ai.RolloutSimulator(seed, P, beta=0.3)
    out = ctl_ref.allocate(sim, P)
    n, c, at = out["n"], out["c"], out["rescued_at"]
    assert n.max() <= 32 and n.sum() == out["generated"] <= 16 * P and out["iterations"] <= 10
    assert ((n - 8) % 2 == 0).all() and (n >= 8).all()
    go = out["group_offsets"]
    params = orc.AdvParams(reject_enable=1, posterior_mode=1)
    ga = orc.group_advantage(out["rewards"], out["lengths"], go, None, params)
    for q in range(P):
        r = out["rewards"][go[q]:go[q + 1]]
        assert int(r.sum()) == c[q] and r.size == n[q]
        if at[q] == 0:
            assert n[q] == 8 and r[:8].sum() > 0
        else:
            assert not r[:8].any()                                  # S = 0: the exploration pass found nothing
            if at[q] > 0:                                           # first success sits in the last increment
                assert n[q] == 8 + 2 * at[q] and not r[:-2].any() and r[-2:].any()
                kept = ga["keep_mask"][go[q]:go[q + 1]]
                assert kept.sum() == 2 * c[q]                       # one incorrect per correct: 2 when c = 1
                a = ga["adv"][go[q]:go[q + 1]][kept > 0]
                assert sorted(np.round(a, 12).tolist()) == [-1.0] * c[q] + [1.0] * c[q]   # Sec. 4.4: a rescued pair gets +-1
            else:
                assert c[q] == 0 and ga["keep_mask"][go[q]:go[q + 1]].sum() == 4   # Strategy 2 keeps 4
    assert (at > 0).any() and (at == 0).any()


@pytest.mark.parametrize("seed,S,n_budget,n_max,k_max,n_extra", [
    (0, 0, 16, 32, 10, 2), (1, 0, 10, 32, 10, 2), (2, 2, 16, 20, 10, 2), (3, 4, 12, 32, 3, 4),
    (4, 0, 16, 12, 10, 2), (5, 1, 9, 32, 10, 3), (6, 0, 8, 32, 10, 2), (7, 3, 16, 32, 0, 2)])
def test_controller_matches_checker(seed, S, n_budget, n_max, k_max, n_extra):
    P = 64
    sim = ai.RolloutSimulator(seed, P, beta=0.4)
    ref = ctl_ref.allocate(sim, P, 8, n_extra, k_max, n_max, n_budget, S)
    got = allocate_rollouts(sim.draw, P, 8, n_extra, k_max, n_max, n_budget, S)
    for key in ("n", "c", "rescued_at", "rewards", "lengths", "group_offsets"):
        assert np.array_equal(getattr(got, key), ref[key]), key
    assert got.generated == ref["generated"] and got.iterations == ref["iterations"]


def test_controller_rejects_inconsistent_budgets():
    sim = ai.RolloutSimulator(0, 4)
    with pytest.raises(ValueError):
        allocate_rollouts(sim.draw, 4, n_explore=8, S=5)
    with pytest.raises(ValueError):
        allocate_rollouts(sim.draw, 4, n_explore=8, n_budget=4)
