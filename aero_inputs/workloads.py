"""Workload recipes: five named configurations plus size overrides for parity tests.

Logits-path workloads (``cfg1``..``cfg3``) carry groups of rollouts with binary
rewards, a token layout (which rollout each token row belongs to, ``-1`` for
right-padding) and a row generator for the logits.  Fused workloads (``cfg4``,
``cfg5``) carry the same group / token structure plus generators for the final
hidden states and the LM-head weight.

Random streams are keyed ``(seed, stream, block)``; tensors with many rows are
drawn in blocks of ``ROWS_PER_BLOCK`` rows so that any block can be regenerated
independently (a checker can draw just the rows it samples) and blocks can be drawn
by several threads at once.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

from .bf16 import f32_to_bf16_bits, f32_to_f16_bits, f32_to_f8e4m3_bits

ROWS_PER_BLOCK = 64

# stream ids (second key of every generator)
_S_STRUCT, _S_REWARD, _S_TARGET, _S_LOGITS, _S_HIDDEN, _S_WEIGHT, _S_OLDLP, _S_PRIO, _S_SIM = range(9)

# Hyper-parameters of the curation step as the paper sets them: 1:k ratio with k=1,
# rescue threshold S=0, tau=1/2, 4 rollouts kept for all-equal groups, Beta(1,1) prior.
ADV_PARAM_DEFAULTS: Dict[str, float] = dict(
    k_ratio=1, s_rescue=0, tau_num=1, tau_den=2, zero_keep=4,
    reject_enable=0, posterior_mode=0, alpha0=1.0, beta0=1.0,
)


def _rng(seed: int, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(stream), int(block)])


def normal_rows(seed: int, stream: int, r0: int, r1: int, ncols: int, sigma: float,
                dtype: str, ld: Optional[int] = None, out: Optional[np.ndarray] = None,
                threads: int = 1) -> np.ndarray:
    """Rows ``[r0, r1)`` of an i.i.d. N(0, sigma^2) matrix with ``ncols`` columns.

    ``dtype`` is ``"f32"`` (float32 values), ``"bf16"`` or ``"f16"`` (uint16 bit patterns, RNE) or
    ``"f8e4m3"`` (uint8 bit patterns, RNE).
    Row ``r`` always comes from block ``r // ROWS_PER_BLOCK`` of the keyed stream, so
    the result does not depend on how the rows are requested.  With ``ld > ncols``
    the trailing columns hold +inf: they are not part of the matrix and a reader that
    touches them is wrong.
    """
    ld = ncols if ld is None else int(ld)
    np_dt = np.float32 if dtype == "f32" else np.uint8 if dtype == "f8e4m3" else np.uint16
    if out is None:
        out = np.empty((r1 - r0, ld), dtype=np_dt)
    assert out.shape == (r1 - r0, ld) and out.dtype == np_dt
    if ld > ncols:
        out[:, ncols:] = (np.inf if dtype == "f32" else np.uint8(0x7F) if dtype == "f8e4m3" else     # f8: NaN
                          np.uint16(0x7F80 if dtype == "bf16" else 0x7C00))

    def do_block(b: int) -> None:
        lo, hi = b * ROWS_PER_BLOCK, (b + 1) * ROWS_PER_BLOCK
        x = _rng(seed, stream, b).standard_normal((ROWS_PER_BLOCK, ncols), dtype=np.float32)
        x *= np.float32(sigma)
        s0, s1 = max(lo, r0), min(hi, r1)
        part = x[s0 - lo:s1 - lo]
        out[s0 - r0:s1 - r0, :ncols] = (part if dtype == "f32" else
                                        f32_to_bf16_bits(part) if dtype == "bf16" else
                                        f32_to_f8e4m3_bits(part) if dtype == "f8e4m3" else f32_to_f16_bits(part))

    blocks = range(r0 // ROWS_PER_BLOCK, (r1 - 1) // ROWS_PER_BLOCK + 1) if r1 > r0 else []
    if threads > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(do_block, blocks))
    else:
        for b in blocks:
            do_block(b)
    return out


def draw_old_logprob(cur_logprob: np.ndarray, seed: int, sigma: float = 0.05,
                     eps_lo: float = 0.2, eps_hi: float = 0.2, margin: float = 5e-3) -> np.ndarray:
    """Behaviour-policy log-probs: the given current log-probs plus N(0, sigma^2) noise.

    The importance ratio the update will see is ``exp(-noise)``.  Any token whose ratio
    falls within ``margin`` of a clip edge ``1-eps_lo`` / ``1+eps_hi`` gets its noise
    redrawn from the same stream, so that a fp32 and a float64 evaluation of the ratio
    cannot land on different sides of the edge.
    """
    cur = np.asarray(cur_logprob, dtype=np.float64)
    rng = _rng(seed, _S_OLDLP)
    noise = rng.normal(0.0, sigma, size=cur.shape)
    for _ in range(64):
        ratio = np.exp(-noise)
        bad = (np.abs(ratio - (1.0 - eps_lo)) < margin) | (np.abs(ratio - (1.0 + eps_hi)) < margin)
        if not bad.any():
            break
        noise[bad] = rng.normal(0.0, sigma, size=int(bad.sum()))
    return (cur + noise).astype(np.float32)


@dataclass
class _Groups:
    """Group / rollout structure shared by both workload kinds."""
    Q: int
    R: int
    group_offsets: np.ndarray      # i32[Q+1]
    rewards: np.ndarray            # f32[R], binary
    lengths: np.ndarray            # i32[R], full valid response length of each rollout
    keep_priority: np.ndarray      # u32[R], random keys for down-sampling
    adv_params: Dict[str, float]


@dataclass
class LogitsWorkload(_Groups):
    name: str = ""
    seed: int = 0
    dtype: str = "bf16"            # "bf16" | "f16" | "f8e4m3" | "f32"
    T: int = 0
    V: int = 0
    ld: int = 0
    sigma: float = 1.0
    eps: float = 0.2
    targets: np.ndarray = field(default=None)        # i32[T]
    token_rollout: np.ndarray = field(default=None)  # i32[T], -1 = padding row

    def logits_rows(self, r0: int, r1: int, threads: int = 1) -> np.ndarray:
        return normal_rows(self.seed, _S_LOGITS, r0, r1, self.V, self.sigma, self.dtype,
                           ld=self.ld, threads=threads)

    def logits_into(self, out: np.ndarray, threads: int = 1) -> np.ndarray:
        return normal_rows(self.seed, _S_LOGITS, 0, self.T, self.V, self.sigma, self.dtype,
                           ld=self.ld, out=out, threads=threads)

    @property
    def n_valid(self) -> int:
        return int((self.token_rollout >= 0).sum())


@dataclass
class FusedWorkload(_Groups):
    name: str = ""
    seed: int = 0
    T: int = 0
    H: int = 0
    V: int = 0
    sigma_h: float = 1.0
    sigma_w: float = 0.02
    eps: float = 0.2
    targets: np.ndarray = field(default=None)
    token_rollout: np.ndarray = field(default=None)

    def hidden_rows(self, r0: int, r1: int, threads: int = 1) -> np.ndarray:
        return normal_rows(self.seed, _S_HIDDEN, r0, r1, self.H, self.sigma_h, "bf16", threads=threads)

    def weight_rows(self, v0: int, v1: int, threads: int = 1) -> np.ndarray:
        return normal_rows(self.seed, _S_WEIGHT, v0, v1, self.H, self.sigma_w, "bf16", threads=threads)

    @property
    def n_valid(self) -> int:
        return int((self.token_rollout >= 0).sum())


# --------------------------------------------------------------------------- structure draws

def _bernoulli_groups(rng, sizes, p_q) -> np.ndarray:
    return np.concatenate([(rng.random(n) < p).astype(np.float32) for n, p in zip(sizes, p_q)]) \
        if len(sizes) else np.zeros(0, np.float32)


def _offsets(sizes) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)


def _packed_layout(rng, group_offsets, lengths, T) -> np.ndarray:
    """Padding-free token layout: groups in a drawn order, their rollouts in order, each
    rollout contributing its tokens until ``T`` rows are filled (the last one is cut
    short; its recorded length stays the full one).  If the rollouts run out first the
    remaining rows are padding (-1)."""
    Q = len(group_offsets) - 1
    tok = np.full(T, -1, np.int32)
    pos = 0
    for q in rng.permutation(Q):
        for i in range(group_offsets[q], group_offsets[q + 1]):
            n = min(int(lengths[i]), T - pos)
            tok[pos:pos + n] = i
            pos += n
            if pos >= T:
                return tok
    return tok


def _padded_layout(lengths, slots) -> np.ndarray:
    """Right-padded layout: rollout ``i`` owns rows ``[i*slots, (i+1)*slots)``."""
    R = len(lengths)
    pos = np.arange(slots, dtype=np.int64)[None, :]
    valid = pos < np.minimum(lengths, slots)[:, None]
    tok = np.where(valid, np.arange(R, dtype=np.int32)[:, None], -1).astype(np.int32)
    return tok.reshape(-1)


def _targets(seed, T, V) -> np.ndarray:
    return _rng(seed, _S_TARGET).integers(0, V, size=T, dtype=np.int32)


def _priority(seed, R) -> np.ndarray:
    return _rng(seed, _S_PRIO).integers(0, 2 ** 32, size=R, dtype=np.uint32)


def _ragged_groups(seed, Q, n_lo, n_hi, len_lo, len_hi, zero_var_frac=None, beta=None):
    """Q groups with sizes U{n_lo..n_hi} and lengths U{len_lo..len_hi}.  Rewards: either
    ``zero_var_frac`` of the groups get all-equal rewards (all 0 or all 1, even odds)
    and the others a count of correct rollouts U{1..n-1} at random positions, or
    Bernoulli(p_q) with p_q ~ Beta(beta, beta)."""
    rs = _rng(seed, _S_STRUCT)
    rr = _rng(seed, _S_REWARD)
    sizes = rs.integers(n_lo, n_hi + 1, size=Q)
    R = int(sizes.sum())
    lengths = rs.integers(len_lo, len_hi + 1, size=R).astype(np.int32)
    if zero_var_frac is not None:
        rewards = []
        for n in sizes:
            r = np.zeros(n, np.float32)
            if rr.random() < zero_var_frac or n < 2:
                r[:] = float(rr.random() < 0.5)
            else:
                c = int(rr.integers(1, n))
                r[rr.permutation(n)[:c]] = 1.0
            rewards.append(r)
        rewards = np.concatenate(rewards)
    else:
        p_q = rr.beta(beta, beta, size=Q)
        rewards = _bernoulli_groups(rr, sizes, p_q)
    return sizes, lengths, rewards, rs


def make_config(name: str, seed: Optional[int] = None, **ov):
    """Build one of the named workloads.

    name   what it is                                            overrides (for smaller parity cases)
    cfg1   4 queries x 8 rollouts x 64 tokens, V=1024, fp32      V, L, ld
    cfg2   2 queries x 8 rollouts, right-padded slots, bf16      V, slots, len_lo, len_hi, ld, dtype
    cfg3   64 curated ragged groups packed into T rows, bf16     V, T, Q, len_lo, len_hi, ld, dtype
    cfg4   fused LM head, H=1536, groups of 8 packed into T      V, T, H, Q, len_lo, len_hi
    cfg5   fused LM head, H=3584, 128 ragged groups packed       V, T, H, Q, len_lo, len_hi
    The default seed is the configuration's ordinal minus one (cfg1 -> 0).
    """
    params = dict(ADV_PARAM_DEFAULTS)
    params.update(ov.pop("adv_params", {}))
    if name == "cfg1":
        seed = 0 if seed is None else seed
        V, L = ov.pop("V", 1024), ov.pop("L", 64)
        Q, N = 4, 8
        sizes = [N] * Q
        rr = _rng(seed, _S_REWARD)
        rewards = _bernoulli_groups(rr, sizes, [0.0, 0.5, 1.0, 0.3])
        lengths = np.full(Q * N, L, np.int32)
        T = Q * N * L
        wl = LogitsWorkload(
            Q=Q, R=Q * N, group_offsets=_offsets(sizes), rewards=rewards, lengths=lengths,
            keep_priority=_priority(seed, Q * N), adv_params=params,
            name=name, seed=seed, dtype="f32", T=T, V=V, ld=ov.pop("ld", V), sigma=2.0,
            targets=_targets(seed, T, V), token_rollout=_padded_layout(lengths, L))
    elif name == "cfg2":
        seed = 1 if seed is None else seed
        V, slots = ov.pop("V", 151936), ov.pop("slots", 1024)
        len_lo, len_hi = ov.pop("len_lo", 128), ov.pop("len_hi", 1024)
        Q, N = 2, 8
        sizes = [N] * Q
        rs, rr = _rng(seed, _S_STRUCT), _rng(seed, _S_REWARD)
        lengths = rs.integers(len_lo, len_hi + 1, size=Q * N).astype(np.int32)
        rewards = _bernoulli_groups(rr, sizes, rr.beta(0.5, 0.5, size=Q))
        T = Q * N * slots
        wl = LogitsWorkload(
            Q=Q, R=Q * N, group_offsets=_offsets(sizes), rewards=rewards, lengths=lengths,
            keep_priority=_priority(seed, Q * N), adv_params=params,
            name=name, seed=seed, dtype=ov.pop("dtype", "bf16"), T=T, V=V, ld=ov.pop("ld", V), sigma=3.0,
            targets=_targets(seed, T, V), token_rollout=_padded_layout(lengths, slots))
    elif name == "cfg3":
        seed = 2 if seed is None else seed
        V, T, Q = ov.pop("V", 151936), ov.pop("T", 32768), ov.pop("Q", 64)
        len_lo, len_hi = ov.pop("len_lo", 64), ov.pop("len_hi", 2048)
        sizes, lengths, rewards, rs = _ragged_groups(seed, Q, 2, 16, len_lo, len_hi, zero_var_frac=0.35)
        go = _offsets(sizes)
        wl = LogitsWorkload(
            Q=Q, R=int(go[-1]), group_offsets=go, rewards=rewards, lengths=lengths,
            keep_priority=_priority(seed, int(go[-1])), adv_params=params,
            name=name, seed=seed, dtype=ov.pop("dtype", "bf16"), T=T, V=V, ld=ov.pop("ld", V), sigma=3.0,
            targets=_targets(seed, T, V), token_rollout=_packed_layout(rs, go, lengths, T))
    elif name in ("cfg4", "cfg5"):
        if name == "cfg4":
            seed = 3 if seed is None else seed
            V, T, H, Q = ov.pop("V", 151936), ov.pop("T", 16384), ov.pop("H", 1536), ov.pop("Q", 8)
            len_lo, len_hi = ov.pop("len_lo", 128), ov.pop("len_hi", 1024)
            n_lo = n_hi = 8
        else:
            seed = 4 if seed is None else seed
            V, T, H, Q = ov.pop("V", 152064), ov.pop("T", 32768), ov.pop("H", 3584), ov.pop("Q", 128)
            len_lo, len_hi = ov.pop("len_lo", 256), ov.pop("len_hi", 4096)
            n_lo, n_hi = 4, 16
        sizes, lengths, rewards, rs = _ragged_groups(seed, Q, n_lo, n_hi, len_lo, len_hi, beta=0.5)
        go = _offsets(sizes)
        wl = FusedWorkload(
            Q=Q, R=int(go[-1]), group_offsets=go, rewards=rewards, lengths=lengths,
            keep_priority=_priority(seed, int(go[-1])), adv_params=params,
            name=name, seed=seed, T=T, H=H, V=V,
            targets=_targets(seed, T, V), token_rollout=_packed_layout(rs, go, lengths, T))
    else:
        raise ValueError(f"unknown workload {name!r}")
    if ov:
        raise TypeError(f"unused overrides for {name}: {sorted(ov)}")
    return wl


# --------------------------------------------------------------------------- one training step

@dataclass
class StepGroups(_Groups):
    """The rollouts of one training step before curation: Q queries x N rollouts each."""
    name: str = "step"
    seed: int = 0


def make_step_groups(seed: int = 5, Q: int = 256, N: int = 16, len_lo: int = 128, len_hi: int = 2048,
                     zero_var_frac: float = 0.35, adv_params: Optional[dict] = None) -> StepGroups:
    """Q groups of N rollouts: ``zero_var_frac`` of the groups have all-equal binary rewards, the
    others a count of correct rollouts U{1..N-1}; response lengths U{len_lo..len_hi}."""
    sizes, lengths, rewards, _ = _ragged_groups(seed, Q, N, N, len_lo, len_hi, zero_var_frac=zero_var_frac)
    go = _offsets(sizes)
    params = dict(ADV_PARAM_DEFAULTS)
    params.update(adv_params or {})
    return StepGroups(Q=Q, R=int(go[-1]), group_offsets=go, rewards=rewards, lengths=lengths,
                      keep_priority=_priority(seed, int(go[-1])), adv_params=params, name="step", seed=seed)


# --------------------------------------------------------------------------- rollout simulator

class RolloutSimulator:
    """Stands in for generation + verification: query q answers correctly with a latent
    probability p_q ~ Beta(beta, beta).  The j-th rollout ever drawn for query q has a fixed
    outcome and length (keyed by (seed, q), position j), so two controllers that ask for the
    same positions see the same rollouts, whatever order they ask in."""

    def __init__(self, seed: int, P: int, max_per_query: int = 32, beta: float = 0.5,
                 len_lo: int = 128, len_hi: int = 2048, p_q: Optional[np.ndarray] = None):
        self.seed, self.P, self.max_per_query = int(seed), int(P), int(max_per_query)
        self.p_q = (_rng(seed, _S_SIM).beta(beta, beta, size=P) if p_q is None
                    else np.asarray(p_q, np.float64).copy())
        assert self.p_q.shape == (P,)
        self.len_lo, self.len_hi = int(len_lo), int(len_hi)

    def draw(self, q: int, start: int, count: int):
        """Rollouts start .. start+count-1 of query q: (rewards f32[count], lengths i32[count])."""
        if start < 0 or count < 0 or start + count > self.max_per_query:
            raise ValueError("rollout positions outside the simulator's range")
        rng = _rng(self.seed, _S_SIM, 1 + int(q))
        u = rng.random(self.max_per_query)
        lengths = rng.integers(self.len_lo, self.len_hi + 1, size=self.max_per_query).astype(np.int32)
        rewards = (u < self.p_q[q]).astype(np.float32)
        return rewards[start:start + count], lengths[start:start + count]
