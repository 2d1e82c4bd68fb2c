"""Float64 CPU checker for the per-token hot path of the group-based RL update.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, by-the-definition
implementation used to check the GPU library and to time a CPU baseline.  It shares
no code with the GPU path, imports nothing but numpy, and nothing in the product
imports it.

Every function takes its inputs at their stored precision (bf16 bit patterns in
uint16 arrays, or float32), widens them exactly to float64, and does all arithmetic
in float64, step by step as the paper states it:

  group_advantage   Eq. 1 (group-relative advantage), Sec. 3.2 (all-equal groups give
                    zero advantage), Sec. 4.1 / Alg. 1 and App. C "Problem
                    Categorization" (strata), Sec. 4.2 Strategy 2 (Beta posterior mean,
                    4 rollouts kept), Strategy 3 (keep all correct + k*c incorrect),
                    Theorem 4.1 (statistics are those of the kept subset), Eq. 2
                    (1/N and 1/|o_i| weights).
  logprob_fwd       App. C softmax policy; log-prob of the sampled token; entropy.
  grpo_loss_bwd     Eq. 2 clipped surrogate (beta = 0) and its gradient w.r.t. the
                    logits, App. A.1 (gradient of the ratio, clipped tokens give zero);
                    optional entropy bonus (Table 8 coefficient) and KL penalty (Eq. 2's beta term).
  lmhead_fused      the same, with logits defined as hidden @ weight^T.

Readings of points the paper leaves open are listed next to the code that takes
them.  Two of them have no external pin ("parity unpinned"): in posterior mode the
standard deviation that divides (r - u~) is taken as sqrt(u~ (1 - u~)); and the entropy
bonus, for which the paper gives a coefficient only, is aggregated with the weights of
Eq. 2 over every token of a weighted rollout (the entropy and its gradient themselves are
pinned).  A third reading of that kind: Eq. 2's KL penalty is evaluated with the per-token
estimator exp(d) - d - 1 of the GRPO literature (the paper names none and trains with beta = 0).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

CAT_ZERO, CAT_PARTIAL, CAT_GOOD, CAT_PERFECT = 0, 1, 2, 3
CAT_RESCUE_BIT = 4          # set when the group is in the rescue stratum (c <= S)
ERR_NONBINARY_REWARD = 1    # bit in the error word
ERR_BAD_TARGET = 2


@dataclass
class AdvParams:
    k_ratio: int = 1          # Strategy 3: m = k * c incorrect rollouts kept, k >= 1
    s_rescue: int = 0         # Strategy 1: rescue threshold S on the count of correct rollouts
    tau_num: int = 1          # tau = tau_num / tau_den = 1/2 splits partial from good
    tau_den: int = 2
    zero_keep: int = 4        # Strategy 2: rollouts kept from an all-equal group
    reject_enable: int = 0    # 0: plain GRPO grouping (keep everything)
    posterior_mode: int = 0   # 0: all-equal groups get zero advantage; 1: Beta posterior mean
    alpha0: float = 1.0
    beta0: float = 1.0


def _f8e4m3_values() -> np.ndarray:
    """The 256 values of the 8-bit float with 4 exponent bits (bias 7) and 3 mantissa bits, in the
    variant without infinities: sign.1111.111 is NaN, every other pattern is finite (largest 448 =
    1.75 * 2^8), exponent field 0 holds zero and the subnormals m * 2^-9."""
    t = np.empty(256, dtype=np.float64)
    for b in range(256):
        e, m = (b >> 3) & 0xF, b & 0x7
        if e == 0xF and m == 0x7:
            v = np.nan
        elif e == 0:
            v = m * 2.0 ** -9
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[b] = -v if b & 0x80 else v
    return t


_F8E4M3 = _f8e4m3_values()


def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values -> float64, exactly.  dtype: "bf16" or "f16" (uint16 bits), "f8e4m3" (uint8 bits),
    "f32", "f64"."""
    if dtype == "f8e4m3":
        x = np.ascontiguousarray(x)
        assert x.dtype == np.uint8
        return _F8E4M3[x]
    if dtype == "bf16":
        x = np.ascontiguousarray(x)
        assert x.dtype == np.uint16
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "f16":      # IEEE binary16: every value is a float64 value
        x = np.ascontiguousarray(x)
        assert x.dtype == np.uint16
        return x.view(np.float16).astype(np.float64)
    return np.asarray(x).astype(np.float64)


# ------------------------------------------------------------------------------------------
# Groups: strata, kept subset, advantages, per-rollout weights
# ------------------------------------------------------------------------------------------

def _smallest(idx, keys, count):
    """`count` members of idx with the smallest (key, index) pairs."""
    order = sorted(idx, key=lambda i: (int(keys[i]), i))
    return order[:count]


def group_advantage(rewards, lengths, group_offsets, keep_priority, p: AdvParams) -> Dict[str, np.ndarray]:
    """Per group q with rollouts [o_q, o_{q+1}):

    1. c = number of rollouts with reward exactly 1, n = group size (binary rewards).
    2. Stratum from the success rate u = c/n with integer compares: Zero (c = 0),
       Perfect (c = n), Partial (0 < u < tau), Good (tau <= u < 1); a separate bit marks
       the rescue stratum u <= S / n, i.e. c <= S.  An empty group counts as Zero.
    3. Kept subset.  Without rejection every rollout is kept.  With rejection: Partial
       keeps all correct rollouts and m = min(k c, n - c) incorrect ones, Good keeps
       everything, Zero / Perfect keep min(zero_keep, n) rollouts in posterior mode and
       nothing otherwise.  "Which ones" is decided by caller-supplied keys: smallest
       (key, index) first; no keys means index order.
    4. Advantages over the kept subset: (r - mean) / std with the population standard
       deviation and no epsilon in the denominator (the proof of Theorem 4.1 uses
       sigma^2 = mu (1 - mu)).
    5. All kept rewards equal (or nothing kept): the group is flagged zero-variance and
       its advantages are 0, or, in posterior mode, (r - u~) / sqrt(u~ (1 - u~)) with
       u~ = (c + alpha0) / (n + alpha0 + beta0) from the observed c and n of the whole
       group.
    6. weight_i = 1 / (Q * n'_q * L_i) for kept rollouts (the 1/N and 1/|o_i| of Eq. 2
       with N the kept group size, and the expectation over queries as the mean over
       all Q groups passed in), 0 for the others.
    """
    rewards = np.asarray(rewards)
    lengths = np.asarray(lengths)
    off = np.asarray(group_offsets).astype(np.int64)
    Q, R = len(off) - 1, len(rewards)
    keys = np.zeros(R, np.uint32) if keep_priority is None else np.asarray(keep_priority)
    r64 = rewards.astype(np.float64)

    adv = np.zeros(R, np.float64)
    weight = np.zeros(R, np.float64)
    keep = np.zeros(R, np.uint8)
    zero_var = np.zeros(Q, np.uint8)
    category = np.zeros(Q, np.uint8)
    err = 0
    curation = bool(p.reject_enable) or bool(p.posterior_mode)

    for q in range(Q):
        idx = list(range(int(off[q]), int(off[q + 1])))
        n = len(idx)
        correct = [i for i in idx if r64[i] == 1.0]
        wrong = [i for i in idx if r64[i] != 1.0]
        if curation and any(r64[i] != 0.0 and r64[i] != 1.0 for i in idx):
            err |= ERR_NONBINARY_REWARD
        c = len(correct)
        if c == 0:
            cat = CAT_ZERO
        elif c == n:
            cat = CAT_PERFECT
        elif c * p.tau_den < n * p.tau_num:
            cat = CAT_PARTIAL
        else:
            cat = CAT_GOOD
        category[q] = cat | (CAT_RESCUE_BIT if c <= p.s_rescue else 0)

        if not p.reject_enable:
            kept = idx
        elif cat == CAT_PARTIAL:
            m = min(p.k_ratio * c, n - c)
            kept = sorted(correct + _smallest(wrong, keys, m))
        elif cat == CAT_GOOD:
            kept = idx
        elif p.posterior_mode:
            kept = sorted(_smallest(idx, keys, min(p.zero_keep, n)))
        else:
            kept = []
        for i in kept:
            keep[i] = 1
        n_kept = len(kept)
        if n_kept == 0:
            zero_var[q] = 1
            continue

        rk = np.array([r64[i] for i in kept])
        if rk.max() == rk.min():
            zero_var[q] = 1
            if p.posterior_mode:
                u = (c + float(p.alpha0)) / (n + float(p.alpha0) + float(p.beta0))
                for i in kept:
                    adv[i] = (r64[i] - u) / np.sqrt(u * (1.0 - u))
        else:
            mu = rk.sum() / n_kept
            sigma = np.sqrt(((rk - mu) ** 2).sum() / n_kept)
            for i in kept:
                adv[i] = (r64[i] - mu) / sigma
        for i in kept:
            if lengths[i] > 0:
                weight[i] = 1.0 / (float(Q) * float(n_kept) * float(lengths[i]))

    kept_index = np.nonzero(keep)[0].astype(np.int32)
    counts = np.array([int(keep[off[q]:off[q + 1]].sum()) for q in range(Q)], np.int64)
    kept_offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    return dict(adv=adv, weight=weight, keep_mask=keep, kept_index=kept_index,
                kept_offsets=kept_offsets, zero_var=zero_var, category=category, err=err)


# ------------------------------------------------------------------------------------------
# Softmax policy: log-prob of the sampled token, entropy, log-partition
# ------------------------------------------------------------------------------------------

def logprob_row(z: np.ndarray, y: int):
    """One row of logits z (float64, already cut to the vocabulary), sampled token y.

    pi = softmax(z) (temperature 1):  lse = log sum_j exp z_j, evaluated as
    m + log sum_j exp(z_j - m) with m = max_j z_j;  log pi(y) = z_y - lse;
    entropy = - sum_j pi_j log pi_j = lse - sum_j pi_j z_j  (natural log).
    """
    m = z.max()
    e = np.exp(z - m)
    s = e.sum()
    lse = m + np.log(s)
    lp = z[y] - lse
    ent = lse - (e * z).sum() / s
    return lp, ent, lse


def logprob_fwd(logits: np.ndarray, dtype: str, V: int, targets, row_active=None):
    """All rows.  logits is [T, ld] at stored precision; columns >= V are not read.
    Rows with row_active == 0 or a negative target give lp = entropy = lse = 0."""
    T = logits.shape[0]
    lp = np.zeros(T)
    ent = np.zeros(T)
    lse = np.zeros(T)
    for t in range(T):
        if (row_active is not None and not row_active[t]) or targets[t] < 0:
            continue
        z = widen(logits[t, :V], dtype)
        lp[t], ent[t], lse[t] = logprob_row(z, int(targets[t]))
    return lp, ent, lse


# ------------------------------------------------------------------------------------------
# Clipped surrogate and its gradient w.r.t. the logits
# ------------------------------------------------------------------------------------------

def token_terms(lp: float, lp_old: float, A: float, w: float, eps_lo: float, eps_hi: float,
                grad_scale: float):
    """One token of a kept rollout with advantage A != 0 and weight w.

    rho = pi(y) / pi_old(y) = exp(lp - lp_old)
    surrogate s = min(rho A, clip(rho, 1 - eps_lo, 1 + eps_hi) A)              (Eq. 2)
    loss term   = - w s                                  (J is maximised; loss = -J)
    d s / d rho = A where the unclipped branch is the smaller one, i.e. rho <= 1 + eps_hi
    for A > 0 and rho >= 1 - eps_lo for A < 0 (equality counts as unclipped), else 0;
    d rho / d lp = rho.  g = d loss / d lp = - grad_scale w A rho [unclipped].
    Returns (loss term, g, unclipped flag, rho).
    """
    rho = np.exp(lp - lp_old)
    clipped_rho = min(max(rho, 1.0 - eps_lo), 1.0 + eps_hi)
    s = min(rho * A, clipped_rho * A)
    unclipped = (rho <= 1.0 + eps_hi) if A > 0 else (rho >= 1.0 - eps_lo)
    g = -grad_scale * w * A * rho if unclipped else 0.0
    return -w * s, g, unclipped, rho


def entropy_grad_row(z: np.ndarray, lse: float, ent: float) -> np.ndarray:
    """d H / d z_j for a softmax policy with H = - sum_j pi_j ln pi_j:
    d pi_k / d z_j = pi_k (1[k = j] - pi_j), hence  d H / d z_j = - pi_j (ln pi_j + H),
    with ln pi_j = z_j - lse."""
    lnp = z - lse
    return -np.exp(lnp) * (lnp + ent)


def grpo_loss_bwd(logits: Optional[np.ndarray], dtype: str, V: int, targets, old_logprob,
                  token_rollout, adv, weight, eps_lo: float, eps_hi: float,
                  grad_scale: float = 1.0, want_dlogits: bool = True,
                  z64: Optional[np.ndarray] = None, entropy_coef: float = 0.0,
                  kl_coef: float = 0.0, ref_logprob=None):
    """loss = - sum_t w_{i(t)} s_t over tokens of kept rollouts, and dlogits.

    A row contributes nothing, and its gradient row is exactly +0, when it is padding
    (token_rollout < 0), has a negative target, or belongs to a rollout with advantage 0
    or weight 0; this is decided before the ratio is looked at.  Otherwise
    dlogits[t, j] = g_t (1[j = y_t] - pi_j)   with pi_j = exp(z_j - lse_t),
    because d log pi(y) / d z_j = 1[j = y] - pi_j for a softmax policy.
    clip_frac = clipped tokens / tokens with a non-zero advantage.

    Entropy bonus (Table 8 gives a coefficient only; aggregation taken to be that of Eq. 2):
    with entropy_coef = c != 0 the objective gains  c sum_t w_{i(t)} H_t  over every token of a
    rollout with w != 0 (whatever its advantage, clipped or not), so
    loss -= c w H_t  and  dlogits[t, j] += - grad_scale c w dH_t/dz_j
                                         = grad_scale c w pi_j (ln pi_j + H_t).

    KL penalty (the - beta D_KL(pi_theta || pi_ref) term inside Eq. 2's token sum; the paper names
    no estimator, the per-token one of the GRPO literature is taken): with kl_coef = beta != 0,
    for every token of a rollout with w != 0 (clipped or not, App. A.1),
        D_t = exp(d) - d - 1,  d = ref_logprob[t] - log pi(y_t)          (>= 0, 0 iff d = 0)
        loss += beta w D_t,    g_t += grad_scale beta w (1 - exp(d))     (d D_t / d log pi = 1 - exp(d)).

    ``z64`` may supply the logits already in float64 ([T, V]) instead of ``logits``.
    """
    T = len(targets)
    adv = np.asarray(adv, np.float64)
    weight = np.asarray(weight, np.float64)
    old_logprob = np.asarray(old_logprob, np.float64)
    eps_lo, eps_hi, grad_scale = float(eps_lo), float(eps_hi), float(grad_scale)
    c_ent, beta = float(entropy_coef), float(kl_coef)
    if beta != 0.0:
        ref_logprob = np.asarray(ref_logprob, np.float64)
    loss = 0.0
    g = np.zeros(T)
    e = np.zeros(T)
    lp = np.zeros(T)
    loss_terms = np.zeros(T)
    dz = np.zeros((T, V)) if want_dlogits else None
    n_signal = n_clipped = 0
    for t in range(T):
        i, y = int(token_rollout[t]), int(targets[t])
        if i < 0 or y < 0 or weight[i] == 0.0 or (adv[i] == 0.0 and c_ent == 0.0 and beta == 0.0):
            continue
        z = z64[t] if z64 is not None else widen(logits[t, :V], dtype)
        lp[t], ent, lse = logprob_row(z, y)
        if adv[i] != 0.0:
            loss_terms[t], g[t], unclipped, _ = token_terms(lp[t], old_logprob[t], adv[i], weight[i],
                                                            eps_lo, eps_hi, grad_scale)
            n_signal += 1
            n_clipped += 0 if unclipped else 1
        if beta != 0.0:
            d = ref_logprob[t] - lp[t]
            loss_terms[t] += beta * weight[i] * (np.exp(d) - d - 1.0)
            g[t] += grad_scale * beta * weight[i] * (1.0 - np.exp(d))
        if c_ent != 0.0:
            loss_terms[t] -= c_ent * weight[i] * ent
            e[t] = grad_scale * c_ent * weight[i]
        loss += loss_terms[t]
        if want_dlogits and (g[t] != 0.0 or e[t] != 0.0):
            row = -g[t] * np.exp(z - lse)
            row[y] += g[t]
            if e[t] != 0.0:
                row -= e[t] * entropy_grad_row(z, lse, ent)
            dz[t] = row
    clip_frac = n_clipped / n_signal if n_signal else 0.0
    return dict(loss=loss, clip_frac=clip_frac, logprob=lp, g=g, e=e, loss_terms=loss_terms, dlogits=dz)


# ------------------------------------------------------------------------------------------
# LM head fused in: logits are hidden @ weight^T (no bias, no soft-cap, temperature 1)
# ------------------------------------------------------------------------------------------

def lmhead_logits(hidden_bits: np.ndarray, weight_bits: np.ndarray) -> np.ndarray:
    """z = h W^T in float64 from bf16 inputs: [T, H] x [V, H]^T -> [T, V]."""
    return widen(hidden_bits, "bf16") @ widen(weight_bits, "bf16").T


def lmhead_fused(hidden_bits, weight_bits, targets, old_logprob=None, token_rollout=None,
                 adv=None, weight=None, eps_lo=0.2, eps_hi=0.2, grad_scale=1.0, entropy_coef=0.0,
                 kl_coef=0.0, ref_logprob=None):
    """Forward statistics of the product logits and, when the loss inputs are given, the
    loss and the gradients dhidden = dz W and dweight = dz^T h with the unrounded dz."""
    z = lmhead_logits(hidden_bits, weight_bits)
    T, V = z.shape
    lp = np.zeros(T)
    ent = np.zeros(T)
    lse = np.zeros(T)
    for t in range(T):
        if targets[t] >= 0:
            lp[t], ent[t], lse[t] = logprob_row(z[t], int(targets[t]))
    out = dict(logprob=lp, entropy=ent, lse=lse)
    if old_logprob is not None:
        b = grpo_loss_bwd(None, "f64", V, targets, old_logprob, token_rollout, adv, weight,
                          eps_lo, eps_hi, grad_scale, want_dlogits=True, z64=z, entropy_coef=entropy_coef,
                          kl_coef=kl_coef, ref_logprob=ref_logprob)
        dz = b["dlogits"]
        out.update(loss=b["loss"], clip_frac=b["clip_frac"], g=b["g"], e=b["e"], loss_terms=b["loss_terms"],
                   dhidden=dz @ widen(weight_bits, "bf16"),
                   dweight=dz.T @ widen(hidden_bits, "bf16"))
    return out
