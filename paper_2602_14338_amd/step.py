"""One policy-update step over a batch of rollout groups, as a sequence of micro-batches.

The step is the part of the group-based RL update that AERO's curation shrinks (Sec. 4): the
curation call decides which rollouts are trained on, the kept rollouts' tokens are packed into
micro-batches of a fixed number of rows, and every micro-batch goes through the loss / gradient
call.  Eq. 2's weights 1/(Q n' |o_i|) are global to the step, so the step's loss is the sum of
the micro-batch losses, and a rollout that is split across two micro-batches keeps its full
length in its weight.

Everything numeric happens in the library calls; this module only does the bookkeeping
(which rollout owns which row of which micro-batch) and the call sequence.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np
import torch

from . import binding
from .binding import AdvParams


@dataclass
class Curation:
    """Device outputs of the curation call for the rollouts of one step."""
    adv: torch.Tensor
    weight: torch.Tensor
    keep_mask: torch.Tensor
    kept_index: torch.Tensor
    kept_offsets: torch.Tensor
    zero_var: torch.Tensor
    category: torch.Tensor
    err: torch.Tensor


def curate(rewards: torch.Tensor, lengths: torch.Tensor, group_offsets: torch.Tensor,
           keep_priority: Optional[torch.Tensor], params: AdvParams) -> Curation:
    """Group advantages, keep set and weights for all rollouts of the step (one library call)."""
    dev = rewards.device
    R, Q = rewards.numel(), group_offsets.numel() - 1
    out = Curation(
        adv=torch.empty(R, device=dev), weight=torch.empty(R, device=dev),
        keep_mask=torch.empty(R, dtype=torch.uint8, device=dev),
        kept_index=torch.empty(R, dtype=torch.int32, device=dev),
        kept_offsets=torch.empty(Q + 1, dtype=torch.int32, device=dev),
        zero_var=torch.empty(Q, dtype=torch.uint8, device=dev),
        category=torch.empty(Q, dtype=torch.uint8, device=dev),
        err=torch.zeros(1, dtype=torch.int32, device=dev))
    binding.aero_group_advantage(rewards, lengths, group_offsets, keep_priority, Q, R, params, out.adv, out.weight,
                                 out.keep_mask, out.kept_index, out.kept_offsets, out.zero_var, out.category,
                                 out.err)
    return out


def plan_microbatches(lengths: np.ndarray, rollouts: np.ndarray, mb_tokens: int) -> np.ndarray:
    """Row ownership of the micro-batches: the tokens of ``rollouts`` (in that order, each with
    its ``lengths`` entry) laid end to end and cut into rows of ``mb_tokens``.  Returns
    int32 [n_mb, mb_tokens] with the owning rollout per row and -1 on the padding at the end of
    the last micro-batch.  A rollout may straddle two micro-batches."""
    if mb_tokens < 1:
        raise ValueError("mb_tokens must be positive")
    rollouts = np.asarray(rollouts, np.int64)
    owner = np.repeat(rollouts.astype(np.int32), np.asarray(lengths, np.int64)[rollouts])
    n_mb = (owner.size + mb_tokens - 1) // mb_tokens
    padded = np.full(n_mb * mb_tokens, -1, np.int32)
    padded[:owner.size] = owner
    return padded.reshape(n_mb, mb_tokens)


def loss_bwd_microbatches(token_rollout: torch.Tensor, logits_of: Callable[[int], torch.Tensor],
                          targets_of: Callable[[int], torch.Tensor], old_logprob_of: Callable[[int], torch.Tensor],
                          dlogits_of: Callable[[int], Optional[torch.Tensor]], adv: torch.Tensor,
                          weight: torch.Tensor, V: int, ld: int, eps_lo: float, eps_hi: float,
                          grad_scale: float = 1.0, entropy_coef: float = 0.0,
                          err_flag: Optional[torch.Tensor] = None, kl_coef: float = 0.0,
                          ref_logprob_of: Optional[Callable[[int], torch.Tensor]] = None) -> torch.Tensor:
    """Runs the loss / gradient call on every micro-batch of ``token_rollout`` ([n_mb, mb_tokens],
    device int32) and returns the per-micro-batch losses (device f32 [n_mb]); their sum is the
    step's loss.  ``*_of(k)`` hand over the tensors of micro-batch k; ``ref_logprob_of`` is needed
    only with a non-zero ``kl_coef`` (Eq. 2's beta)."""
    n_mb, mb_tokens = token_rollout.shape
    dev = token_rollout.device
    R = adv.numel()
    losses = torch.zeros(max(n_mb, 1), device=dev)
    ws = torch.empty(max(binding.aero_workspace_bytes(binding.OP_GRPO_LOSS_BWD, T=mb_tokens, V=V, R=R), 1),
                     dtype=torch.uint8, device=dev)
    for k in range(n_mb):
        binding.aero_grpo_loss_bwd(logits_of(k), mb_tokens, V, ld, targets_of(k), None, old_logprob_of(k),
                                   token_rollout[k], adv, weight, R, eps_lo, eps_hi, grad_scale, losses[k:k + 1],
                                   None, None, dlogits_of(k), ws, err_flag, entropy_coef=entropy_coef,
                                   kl_coef=kl_coef,
                                   ref_logprob=ref_logprob_of(k) if ref_logprob_of is not None else None)
    return losses[:n_mb]
