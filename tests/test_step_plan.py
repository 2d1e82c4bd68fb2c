"""Host bookkeeping of the step driver: which rollout owns which micro-batch row (CPU only)."""
import numpy as np
import pytest

from paper_2602_14338_amd.step import plan_microbatches


def test_rows_follow_the_rollout_order_and_lengths():
    lengths = np.array([3, 5, 2, 4], np.int32)
    plan = plan_microbatches(lengths, np.array([2, 0, 3]), 4)
    assert plan.dtype == np.int32 and plan.shape == (3, 4)
    assert plan.reshape(-1).tolist() == [2, 2, 0, 0, 0, 3, 3, 3, 3, -1, -1, -1]


def test_a_rollout_may_straddle_micro_batches_and_counts_are_kept():
    rng = np.random.default_rng(0)
    lengths = rng.integers(1, 50, size=40).astype(np.int32)
    rollouts = rng.permutation(40)[:23]
    plan = plan_microbatches(lengths, rollouts, 16)
    flat = plan.reshape(-1)
    valid = flat[flat >= 0]
    assert valid.size == lengths[rollouts].sum() and (flat[valid.size:] == -1).all()
    for i in rollouts:
        assert (valid == i).sum() == lengths[i]
    # order of first appearance is the order given
    _, first = np.unique(valid, return_index=True)
    assert valid[np.sort(first)].tolist() == rollouts.tolist()
    assert any(len(set(np.nonzero((plan == i).any(axis=1))[0])) > 1 for i in rollouts)


def test_nothing_kept_gives_no_micro_batch():
    plan = plan_microbatches(np.array([4, 4], np.int32), np.zeros(0, np.int64), 8)
    assert plan.shape == (0, 8)
    with pytest.raises(ValueError):
        plan_microbatches(np.array([4], np.int32), np.array([0]), 0)
