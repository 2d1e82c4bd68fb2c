"""Plumbing for the GPU parity tests: upload workloads, call the C ABI through the binding,
bring results back as float64 / integer numpy arrays.  No arithmetic of the method here."""
import numpy as np
import torch

import paper_2602_14338_amd as aero
from paper_2602_14338_amd import binding

DEV = "cuda:0"


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)


def logits_to_dev(arr, dtype):
    """Host logits (float32 values, bf16 / fp16 bit patterns in uint16, 8-bit float patterns in uint8)
    -> device tensor."""
    if dtype == "f8e4m3":
        return torch.from_numpy(arr).to(DEV).view(torch.float8_e4m3fn)
    if dtype in ("bf16", "f16"):
        return torch.from_numpy(arr.view(np.int16)).to(DEV).view(torch.bfloat16 if dtype == "bf16" else torch.float16)
    return torch.from_numpy(arr).to(DEV)


def to_np64(t):
    if t.dtype == torch.float8_e4m3fn:     # widened on the host by the checker's table
        from oracle import aero_oracle as orc
        return orc.widen(t.view(torch.uint8).cpu().numpy(), "f8e4m3")
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy().astype(np.float64)


SEVEN_F8 = 0x4E    # 7.0 = 1.75 * 2^2 in the 8-bit float format


def raw_bits(t):
    """Integer view of a stored tensor (for indexing and bit comparisons; some 8-bit float kernels
    of the tensor library may be missing, integer ones are not)."""
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8)
    return t.view(torch.int32) if t.dtype == torch.float32 else t.view(torch.int16)


def full_like_seven(t):
    """A buffer of the same shape and type filled with 7.0 (to see what a call leaves unwritten)."""
    if t.dtype == torch.float8_e4m3fn:
        return torch.full(t.shape, SEVEN_F8, dtype=torch.uint8, device=t.device).view(torch.float8_e4m3fn)
    return torch.full_like(t, 7.0)


def all_seven(t):
    if t.dtype == torch.float8_e4m3fn:
        return bool((t.view(torch.uint8) == SEVEN_F8).all())
    return bool((t.float() == 7.0).all())


def run_group_advantage(wl_or_arrays, params: dict, keys="wl"):
    if isinstance(wl_or_arrays, tuple):
        rewards, lengths, offsets, kp = wl_or_arrays
    else:
        wl = wl_or_arrays
        rewards, lengths, offsets, kp = wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority
    if keys is None:
        kp = None
    Q, R = len(offsets) - 1, len(rewards)
    d = dict(
        adv=torch.full((R,), 7.0, device=DEV), weight=torch.full((R,), 7.0, device=DEV),
        keep_mask=torch.full((R,), 9, dtype=torch.uint8, device=DEV),
        kept_index=torch.full((R,), -5, dtype=torch.int32, device=DEV),
        kept_offsets=torch.full((Q + 1,), -5, dtype=torch.int32, device=DEV),
        zero_var=torch.full((Q,), 9, dtype=torch.uint8, device=DEV),
        category=torch.full((Q,), 9, dtype=torch.uint8, device=DEV),
        err=torch.zeros(1, dtype=torch.int32, device=DEV))
    aero.aero_group_advantage(dev(rewards.astype(np.float32)), dev(lengths.astype(np.int32)),
                              dev(offsets.astype(np.int32)),
                              dev(kp.astype(np.uint32).view(np.int32)) if kp is not None else None,
                              Q, R, aero.AdvParams(**params), d["adv"], d["weight"], d["keep_mask"],
                              d["kept_index"], d["kept_offsets"], d["zero_var"], d["category"], d["err"])
    torch.cuda.synchronize()
    return d


def run_fwd(logits_d, T, V, ld, targets, row_active=None, want_entropy=True):
    lp = torch.full((T,), 7.0, device=DEV)
    ent = torch.full((T,), 7.0, device=DEV) if want_entropy else None
    lse = torch.full((T,), 7.0, device=DEV)
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    aero.aero_logprob_fwd(logits_d, T, V, ld, dev(targets), dev(row_active) if row_active is not None else None,
                          lp, ent, lse, err)
    torch.cuda.synchronize()
    return lp, ent, lse, int(err.item())


def run_loss_bwd(logits_d, T, V, ld, targets, lse_d, old_lp, token_rollout, adv, weight, eps=0.2,
                 grad_scale=1.0, inplace=False, want_dlogits=True, stats=False, entropy_coef=0.0, entropy=None,
                 kl_coef=0.0, ref_logprob=None):
    R = len(adv)
    ws_bytes = aero.aero_workspace_bytes(binding.OP_GRPO_LOSS_BWD, T=T, V=V, R=R)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device=DEV)
    loss = torch.full((1,), 7.0, device=DEV)
    clip = torch.full((1,), 7.0, device=DEV)
    lp_out = torch.full((T,), 7.0, device=DEV)
    if not want_dlogits:
        dl = None
    elif inplace:
        dl = logits_d
    else:
        dl = full_like_seven(logits_d)
    err = torch.zeros(1, dtype=torch.int32, device=DEV)
    ent_out = torch.full((T,), 7.0, device=DEV) if stats else None
    lse_out = torch.full((T,), 7.0, device=DEV) if stats else None
    aero.aero_grpo_loss_bwd(logits_d, T, V, ld, dev(targets), lse_d, dev(old_lp.astype(np.float32)),
                            dev(token_rollout), dev(adv.astype(np.float32)), dev(weight.astype(np.float32)), R,
                            eps, eps, grad_scale, loss, clip, lp_out, dl, ws, err, entropy_out=ent_out,
                            lse_out=lse_out, entropy_coef=entropy_coef,
                            entropy=dev(entropy.astype(np.float32)) if entropy is not None else None,
                            kl_coef=kl_coef,
                            ref_logprob=dev(ref_logprob.astype(np.float32)) if ref_logprob is not None else None)
    torch.cuda.synchronize()
    return dict(loss=loss, clip_frac=clip, logprob=lp_out, dlogits=dl, err=int(err.item()), entropy=ent_out,
                lse=lse_out)


# Loss tolerance.  Stated for the method: 1e-4 relative.  It is applied as stated whenever the
# reference is well conditioned: sum_t |term_t| <= CANCEL_RATIO_STRICT * |loss|.  With
# group-standardised advantages (Eq. 1) the per-token terms of Eq. 2 cancel almost exactly when the
# ratio is near 1, so the total can be orders of magnitude smaller than its terms; each term
# carries the fp32 rounding of its log-probability (an ulp of a value near 10 is about 1e-6), and
# that error does not shrink with the total.  Only in that case (ratio above the threshold) the
# bound gains 2^-22 * sum_t |term_t|.
CANCEL_RATIO_STRICT = 16.0


def cancel_ratio(loss_ref, loss_terms):
    total = float(np.abs(np.asarray(loss_terms, np.float64)).sum())
    return total / abs(float(loss_ref)) if float(loss_ref) != 0.0 else (np.inf if total > 0 else 0.0)


def loss_bound(loss_ref, loss_terms):
    """Allowed |loss - loss_ref| (see the comment above)."""
    strict = 1e-4 * abs(float(loss_ref))
    if cancel_ratio(loss_ref, loss_terms) <= CANCEL_RATIO_STRICT:
        return strict
    return strict + 2.0 ** -22 * float(np.abs(np.asarray(loss_terms, np.float64)).sum())


def assert_loss(got, loss_ref, loss_terms, strict=False):
    """strict=True: the case is meant to be well conditioned, so the pure 1e-4 relative bound
    must be the one in force."""
    ratio = cancel_ratio(loss_ref, loss_terms)
    if strict:
        assert ratio <= CANCEL_RATIO_STRICT, "not a well-conditioned case: sum|term| / |loss| = %.3g" % ratio
    bound = loss_bound(loss_ref, loss_terms)
    diff = abs(float(got) - float(loss_ref))
    assert diff <= bound, ("loss %.9e, reference %.9e: |diff| %.3e > bound %.3e (%s; sum|term| / |loss| = %.3g)"
                           % (float(got), float(loss_ref), diff, bound,
                              "1e-4 relative" if ratio <= CANCEL_RATIO_STRICT else "1e-4 relative + 2^-22 sum|term|",
                              ratio))
    return ratio
