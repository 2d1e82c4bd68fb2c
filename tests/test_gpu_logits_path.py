"""GPU parity for the logits path: group advantages, softmax statistics, clipped loss and
dlogits, each compared element by element with the float64 checker on the same seeded inputs.

Tolerances (stated for the method): masks, kept indices and counts bit-exact; log-probs and
entropy within 2e-3 absolute; loss within 1e-4 relative; dlogits within 1e-2 absolute and,
because |dlogits| <= |g_t| is tiny, also scale-free: within 1e-2 |g_t| plus one bf16 / fp32
rounding of the entry.  Advantages and weights within 1e-6 relative.
"""
import numpy as np
import pytest
import torch

import aero_inputs as ai
from oracle import aero_oracle as orc
from oracle.aero_oracle import AdvParams

pytestmark = pytest.mark.gpu

LP_TOL = 2e-3
ENT_TOL = 2e-3
DZ_ATOL = 1e-2


@pytest.fixture(scope="module")
def gh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_helpers
    return gpu_helpers


# ------------------------------------------------------------------ group advantage

MODES = [dict(), dict(reject_enable=1), dict(reject_enable=1, posterior_mode=1), dict(posterior_mode=1),
         dict(reject_enable=1, k_ratio=2), dict(reject_enable=1, k_ratio=3, s_rescue=1, zero_keep=2,
                                                posterior_mode=1, alpha0=0.5, beta0=2.0)]


def check_groups(gh, arrays, params, keys="wl"):
    rewards, lengths, offsets, kp = arrays
    ref = orc.group_advantage(rewards, lengths, offsets, kp if keys else None, AdvParams(**params))
    out = gh.run_group_advantage(arrays, params, keys=keys)
    nk = int(ref["kept_offsets"][-1])
    assert np.array_equal(out["keep_mask"].cpu().numpy(), ref["keep_mask"])
    assert np.array_equal(out["kept_offsets"].cpu().numpy(), ref["kept_offsets"])
    assert np.array_equal(out["kept_index"].cpu().numpy()[:nk], ref["kept_index"])
    assert np.array_equal(out["zero_var"].cpu().numpy(), ref["zero_var"])
    assert np.array_equal(out["category"].cpu().numpy(), ref["category"])
    assert int(out["err"].item()) == ref["err"]
    for k in ("adv", "weight"):
        got = out[k].cpu().numpy().astype(np.float64)
        assert np.allclose(got, ref[k], rtol=1e-6, atol=0), k
        assert np.array_equal(got == 0, ref[k] == 0), k
    return ref, out


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
@pytest.mark.parametrize("mode", range(len(MODES)))
def test_group_advantage_configs(gh, name, mode):
    wl = ai.make_config(name)
    check_groups(gh, (wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority), MODES[mode])


def test_group_advantage_edge_cases(gh):
    rng = np.random.default_rng(21)
    # big groups (several strides of 64), empty groups, single-rollout groups, tied keys, no keys
    sizes = [0, 1, 200, 0, 65, 64, 2, 3, 129, 0]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    R = int(off[-1])
    rewards = (rng.random(R) < 0.2).astype(np.float32)
    rewards[off[5]:off[6]] = 1.0
    lengths = rng.integers(0, 50, size=R).astype(np.int32)       # includes zero lengths
    keys = rng.integers(0, 3, size=R).astype(np.uint32)
    for params in MODES:
        check_groups(gh, (rewards, lengths, off, keys), params)
        check_groups(gh, (rewards, lengths, off, keys), params, keys=None)
    # Q = 0 and R = 0
    out = gh.run_group_advantage((np.zeros(0, np.float32), np.zeros(0, np.int32), np.array([0], np.int32), None),
                                 dict(), keys=None)
    assert out["kept_offsets"].cpu().tolist() == [0]
    # many groups: the scan spans several entries per thread
    sizes = rng.integers(0, 6, size=5000)
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    R = int(off[-1])
    rewards = (rng.random(R) < 0.4).astype(np.float32)
    check_groups(gh, (rewards, rng.integers(1, 9, size=R).astype(np.int32), off,
                      rng.integers(0, 2 ** 32, size=R, dtype=np.uint32)), dict(reject_enable=1, posterior_mode=1))


@pytest.mark.parametrize("seed", range(16))
def test_group_advantage_random_structures(gh, seed):
    """Seeded random group structures (empty, single, several strides of 64 wide), success rates, tied keys
    and hyper-parameters of the curation step, all outputs bit for bit / to 1e-6 against the checker."""
    rng = np.random.default_rng(1000 + seed)
    Q = int(rng.integers(1, 300))
    sizes = np.where(rng.random(Q) < 0.1, rng.integers(65, 200, size=Q), rng.integers(0, 34, size=Q))
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    R = int(off[-1])
    p_q = np.repeat(rng.beta(0.5, 0.5, size=Q), sizes)
    rewards = (rng.random(R) < p_q).astype(np.float32)
    lengths = rng.integers(1, 3000, size=R).astype(np.int32)
    keys = rng.integers(0, int(rng.choice([2, 5, 2 ** 32])), size=R).astype(np.uint32)
    tau = [(1, 2), (1, 3), (2, 3), (1, 1)][int(rng.integers(4))]
    params = dict(k_ratio=int(rng.integers(1, 5)), s_rescue=int(rng.integers(0, 4)), tau_num=tau[0], tau_den=tau[1],
                  zero_keep=int(rng.integers(1, 7)), reject_enable=int(rng.integers(2)),
                  posterior_mode=int(rng.integers(2)), alpha0=float(rng.choice([0.5, 1.0, 2.0])),
                  beta0=float(rng.choice([0.5, 1.0, 3.0])))
    check_groups(gh, (rewards, lengths, off, keys), params)
    check_groups(gh, (rewards, lengths, off, keys), params, keys=None)


def test_group_advantage_general_rewards_and_error_flag(gh):
    rng = np.random.default_rng(22)
    sizes = [5, 9, 16, 70]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    rewards = rng.normal(size=int(off[-1])).astype(np.float32)
    rewards[off[1]:off[2]] = 0.25                                    # all equal, non-binary
    arrays = (rewards, np.full(len(rewards), 11, np.int32), off, None)
    ref = orc.group_advantage(*arrays, AdvParams())
    out = gh.run_group_advantage(arrays, dict(), keys=None)
    assert np.allclose(out["adv"].cpu().numpy(), ref["adv"], rtol=2e-6, atol=1e-7)
    assert out["zero_var"].cpu().tolist() == [0, 1, 0, 0] and int(out["err"].item()) == 0
    out = gh.run_group_advantage(arrays, dict(reject_enable=1), keys=None)
    assert int(out["err"].item()) & orc.ERR_NONBINARY_REWARD


# ------------------------------------------------------------------ softmax statistics

def check_fwd(gh, wl, row_active=None, targets=None, offset_elems=0):
    targets = wl.targets if targets is None else targets
    host = wl.logits_rows(0, wl.T)
    ref = orc.logprob_fwd(host, wl.dtype, wl.V, targets, row_active)
    if offset_elems:   # misaligned base pointer: slice a flat buffer
        flat = np.concatenate([np.zeros(offset_elems, host.dtype), host.reshape(-1)])
        d = gh.logits_to_dev(flat, wl.dtype)[offset_elems:]
    else:
        d = gh.logits_to_dev(host, wl.dtype)
    lp, ent, lse, err = gh.run_fwd(d, wl.T, wl.V, wl.ld, targets, row_active)
    ignored = targets < 0
    if row_active is not None:
        ignored |= row_active == 0
    for got, want, tol in ((lp, ref[0], LP_TOL), (ent, ref[1], ENT_TOL), (lse, ref[2], LP_TOL)):
        g = got.cpu().numpy().astype(np.float64)
        assert np.isfinite(g).all()
        assert np.abs(g - want).max() <= tol
        assert not g[ignored].any()                 # ignored rows give exact zeros
    return err


def test_fwd_cfg1_full(gh):
    assert check_fwd(gh, ai.make_config("cfg1")) == 0


@pytest.mark.parametrize("V,ld", [(1000, 1000), (1000, 1008), (4999, 4999), (4999, 5008), (32768, 32768),
                                  (151936, 151936), (152064, 152064), (262144, 262152), (7, 8), (1, 1), (65, 72)])
def test_fwd_bf16_shapes(gh, V, ld):
    slots = 4 if V > 100000 else 12
    wl = ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots)
    active = (wl.token_rollout >= 0).astype(np.uint8)
    assert check_fwd(gh, wl) == 0
    assert check_fwd(gh, wl, row_active=active) == 0


@pytest.mark.parametrize("V,ld", [(1024, 1024), (1023, 1023), (5000, 5004), (151936, 151936)])
def test_fwd_f32_shapes(gh, V, ld):
    wl = ai.make_config("cfg1", V=V, ld=ld, L=2)
    assert check_fwd(gh, wl) == 0


# fp16 storage (beyond the paper's bf16 runs, App. C): same definitions on binary16 values, the
# checker widens them exactly.  "Parity unpinned" by the paper in the sense that no experiment of
# it uses this format; the arithmetic is the pinned one.
@pytest.mark.parametrize("V,ld", [(1000, 1000), (4999, 5008), (151936, 151936), (65, 72), (7, 8)])
def test_fwd_f16_shapes(gh, V, ld):
    slots = 4 if V > 100000 else 12
    wl = ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots, dtype="f16")
    active = (wl.token_rollout >= 0).astype(np.uint8)
    assert check_fwd(gh, wl) == 0
    assert check_fwd(gh, wl, row_active=active) == 0
    assert check_fwd(gh, wl, offset_elems=3) == 0          # misaligned base: scalar path


# 8-bit float storage (4 exponent, 3 mantissa bits).  Parity unpinned by the paper (it trains in bf16,
# App. C); the arithmetic is the pinned one, the widening is pinned bit for bit on the host.
@pytest.mark.parametrize("V,ld", [(1000, 1008), (4999, 5008), (151936, 151936), (65, 80), (7, 16), (5000, 5003)])
def test_fwd_f8_shapes(gh, V, ld):
    slots = 4 if V > 100000 else 12
    wl = ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots, dtype="f8e4m3")
    active = (wl.token_rollout >= 0).astype(np.uint8)
    assert check_fwd(gh, wl) == 0
    assert check_fwd(gh, wl, row_active=active) == 0
    assert check_fwd(gh, wl, offset_elems=3) == 0          # misaligned base: scalar path


def test_fwd_misaligned_base_and_bad_targets(gh):
    wl = ai.make_config("cfg2", V=4096, slots=6, len_lo=1, len_hi=6)
    assert check_fwd(gh, wl, offset_elems=3) == 0
    tg = wl.targets.copy()
    tg[::5] = -1
    assert check_fwd(gh, wl, targets=tg) == 0
    tg[1] = wl.V          # outside the vocabulary: ignored row + error bit, no fault
    tg[2] = 2 ** 31 - 1
    host = wl.logits_rows(0, wl.T)
    lp, ent, lse, err = gh.run_fwd(gh.logits_to_dev(host, "bf16"), wl.T, wl.V, wl.ld, tg)
    assert err & 2 and lp[1].item() == 0 and lse[2].item() == 0
    assert torch.isfinite(lp).all()


def test_fwd_large_magnitudes(gh):
    """Rows whose maximum moves a lot along the row and logits far outside exp's fp32 range."""
    V = 20000
    rng = np.random.default_rng(31)
    z = rng.normal(0, 3, size=(6, V)).astype(np.float32)
    z[0] += np.linspace(-300, 300, V, dtype=np.float32)       # maximum at the very end
    z[1] += np.linspace(300, -300, V, dtype=np.float32)       # maximum at the start
    z[2] *= 100.0
    z[3] = 5.0                                                # uniform row
    z[4, :] = -200.0
    z[4, 77] = 200.0                                          # one dominant logit
    z[5] -= 5000.0
    tg = np.array([V - 1, 0, 5, 6, 77, 9], np.int32)
    for dtype in ("f32", "bf16"):
        host = z if dtype == "f32" else ai.f32_to_bf16_bits(z)
        ref = orc.logprob_fwd(host, dtype, V, tg)
        lp, ent, lse, err = gh.run_fwd(gh.logits_to_dev(host, dtype), 6, V, V, tg)
        scale = np.maximum(1.0, np.abs(ref[2]))
        assert (np.abs(lp.cpu().numpy() - ref[0]) <= LP_TOL * scale).all()
        assert (np.abs(lse.cpu().numpy() - ref[2]) <= LP_TOL * scale).all()
        assert (np.abs(ent.cpu().numpy() - ref[1]) <= ENT_TOL * scale).all()


def test_fwd_empty(gh):
    z = torch.zeros((0, 16), dtype=torch.bfloat16, device=gh.DEV)
    gh.run_fwd(z, 0, 16, 16, np.zeros(0, np.int32))


# ------------------------------------------------------------------ loss and dlogits

def elt_rounding(dtype, ref_abs):
    """One rounding of the stored gradient entry: bf16 has 8 significant bits, fp32 24, fp16 11
    and a fixed grid of 2^-24 below 2^-14 (subnormals), the 8-bit float 4 and a grid of 2^-9 below 2^-6."""
    if dtype == "f16":
        return ref_abs * 2.0 ** -11 + 2.0 ** -25
    if dtype == "f8e4m3":
        return ref_abs * 2.0 ** -4 + 2.0 ** -10
    return ref_abs * (2.0 ** -8 if dtype == "bf16" else 2.0 ** -23) + 1e-30


def check_loss_bwd(gh, wl, params, sigma_old=0.05, use_oracle_lse=True, inplace=False, grad_scale=1.0,
                   expect_clip=False, stats=False, entropy_coef=0.0, kl_coef=0.0, adv_map=None, strict_loss=False,
                   untouched=None):
    """adv_map: replaces the group-relative advantages by adv_map(adv) before both sides see them
    (supplied advantages; e.g. abs makes every term of the loss carry one sign).
    strict_loss: the loss must meet the pure 1e-4 relative bound (well-conditioned case).
    untouched: "half" or "all" - that share of the padding rows is handed to the library as
    AERO_ROW_UNTOUCHED; their gradient rows must keep what the buffer held before the call, everything
    else must come out as for plain padding (the checker sees plain padding)."""
    host = wl.logits_rows(0, wl.T)
    tr_gpu = wl.token_rollout.copy()
    chosen = np.zeros(0, dtype=np.int64)
    if untouched is not None:
        pads = np.flatnonzero(wl.token_rollout < 0)
        chosen = pads if untouched == "all" else pads[::2]
        assert chosen.size > 0
        tr_gpu[chosen] = gh.binding.AERO_ROW_UNTOUCHED
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams(**params))
    if adv_map is not None:
        ga["adv"] = adv_map(ga["adv"].astype(np.float32)).astype(np.float64)
    active = (wl.token_rollout >= 0).astype(np.uint8)
    lp_ref, ent_ref, lse_ref = orc.logprob_fwd(host, wl.dtype, wl.V, wl.targets, active)
    old = ai.draw_old_logprob(lp_ref, wl.seed, sigma=sigma_old)
    eps = np.float32(wl.eps)
    # log-probs of a reference policy: the behaviour ones moved by seeded noise (input data only)
    ref_lp = (old + np.random.default_rng(wl.seed + 77).normal(0, 0.2, size=old.shape)).astype(np.float32) \
        if kl_coef != 0.0 else None
    ref = orc.grpo_loss_bwd(host, wl.dtype, wl.V, wl.targets, old, wl.token_rollout, ga["adv"].astype(np.float32),
                            ga["weight"].astype(np.float32), eps, eps, grad_scale, entropy_coef=entropy_coef,
                            kl_coef=kl_coef, ref_logprob=ref_lp)
    d = gh.logits_to_dev(host, wl.dtype)
    lse_d = gh.dev(lse_ref.astype(np.float32)) if use_oracle_lse else None
    before = gh.raw_bits(d)[torch.from_numpy(chosen).to(gh.DEV)].clone() if (inplace and chosen.size) else None
    out = gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, wl.targets, lse_d, old, tr_gpu,
                          ga["adv"], ga["weight"], eps=float(eps), grad_scale=grad_scale, inplace=inplace, stats=stats,
                          entropy_coef=entropy_coef,
                          entropy=ent_ref if (use_oracle_lse and entropy_coef != 0.0) else None,
                          kl_coef=kl_coef, ref_logprob=ref_lp)
    assert out["err"] == 0
    loss = out["loss"].item()
    gh.assert_loss(loss, ref["loss"], ref["loss_terms"], strict=strict_loss)
    assert abs(out["clip_frac"].item() - ref["clip_frac"]) < 1e-6
    if expect_clip:
        assert 0.02 < ref["clip_frac"] < 0.98
    lp = out["logprob"].cpu().numpy().astype(np.float64)
    if stats:   # statistics for every valid row, as the forward call would give them
        assert np.abs(lp - lp_ref).max() <= LP_TOL and not lp[active == 0].any()
        for key, want in (("entropy", ent_ref), ("lse", lse_ref)):
            got = out[key].cpu().numpy().astype(np.float64)
            assert np.abs(got - want).max() <= LP_TOL and not got[active == 0].any()
    else:
        assert np.abs(lp - ref["logprob"]).max() <= LP_TOL
    dz = gh.to_np64(out["dlogits"])[:, :wl.V]
    want = ref["dlogits"]
    if chosen.size:   # not written at all: the rows hold what the buffer held before the call
        rows = gh.raw_bits(out["dlogits"])[torch.from_numpy(chosen).to(gh.DEV)]
        if inplace:
            assert torch.equal(rows, before)
        else:
            assert torch.equal(rows, gh.raw_bits(gh.full_like_seven(out["dlogits"][:1])).expand_as(rows))
        dz[chosen] = 0.0
    assert np.isfinite(dz).all()
    # stated for the unscaled gradient; an 8-bit stored entry's own rounding (2^-4 relative) is allowed on top
    stored = elt_rounding(wl.dtype, np.abs(want)) if wl.dtype == "f8e4m3" else 0.0
    assert (np.abs(dz - want) <= DZ_ATOL * max(1.0, grad_scale) + stored).all()
    # scale of a row: |g_t| for the surrogate, |e_t| (|p ln p| + p H_t) <= |e_t| (1 + H_t) for the entropy term
    scale = np.abs(ref["g"]) + np.abs(ref["e"]) * (1.0 + ent_ref)
    bound = 1e-2 * scale[:, None] + elt_rounding(wl.dtype, np.abs(want))
    assert (np.abs(dz - want) <= bound).all()
    dead = (ref["g"] == 0) & (ref["e"] == 0)
    dead[chosen] = False
    bits = gh.raw_bits(out["dlogits"])[:, :wl.V]
    assert not bits[torch.from_numpy(dead).to(gh.DEV)].any()       # exactly +0, sign bit included
    if wl.ld > wl.V and not inplace:                                # pad columns are not written
        assert gh.all_seven(out["dlogits"][:, wl.V:])
    return ref, out


def test_loss_bwd_cfg1_full(gh):
    wl = ai.make_config("cfg1")
    ref, _ = check_loss_bwd(gh, wl, dict())
    assert (ref["g"] == 0).sum() >= 2 * 8 * 64      # the two all-equal groups
    check_loss_bwd(gh, wl, dict(), use_oracle_lse=False)
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, expect_clip=True)
    check_loss_bwd(gh, wl, dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, inplace=True, grad_scale=64.0)


def test_entropy_bonus_cfg1(gh):
    """Entropy bonus (Table 8 coefficient and a large one): rows of the all-equal groups now
    carry the entropy-only gradient, rows of dropped rollouts stay exactly +0."""
    wl = ai.make_config("cfg1")
    ref0, _ = check_loss_bwd(gh, wl, dict())
    for coef in (1e-3, 0.05):
        ref, _ = check_loss_bwd(gh, wl, dict(), entropy_coef=coef)
        assert (ref["e"] != 0).sum() > (ref0["g"] != 0).sum() and ref["loss"] < ref0["loss"]
        assert ((ref["g"] == 0) & (ref["e"] != 0)).any()
        check_loss_bwd(gh, wl, dict(), use_oracle_lse=False, sigma_old=0.3, expect_clip=True, entropy_coef=coef,
                       grad_scale=16.0)
    # curation drops rollouts (weight 0): their rows have neither term
    ref, _ = check_loss_bwd(gh, wl, dict(reject_enable=1, posterior_mode=1), entropy_coef=0.01, inplace=True)
    assert ((ref["e"] == 0) & (wl.token_rollout >= 0)).any()


# 151936 and 32768 take the single-pass kernels (streaming / one workgroup per row) when lse is not given
@pytest.mark.parametrize("V,ld,slots", [(151936, 151936, 6), (32768, 32768, 8), (4999, 4999, 10), (1000, 1008, 10)])
def test_entropy_bonus_cfg2_reduced(gh, V, ld, slots):
    wl = ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots)
    check_loss_bwd(gh, wl, dict(), entropy_coef=1e-3)
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, use_oracle_lse=False, expect_clip=True, entropy_coef=0.02, stats=True)


@pytest.mark.parametrize("cfg,kw", [("cfg1", dict()), ("cfg2", dict(V=151936, ld=151936, slots=6, len_lo=1, len_hi=6)),
                                    ("cfg2", dict(V=32768, ld=32768, slots=8, len_lo=1, len_hi=8)),
                                    ("cfg2", dict(V=4999, ld=4999, slots=10, len_lo=1, len_hi=10))])
def test_kl_penalty(gh, cfg, kw):
    """Eq. 2's beta term: every token of a weighted rollout is pulled towards the reference policy,
    also in the all-equal groups and on clipped tokens; alone and together with the entropy bonus."""
    wl = ai.make_config(cfg, **kw)
    ref0, _ = check_loss_bwd(gh, wl, dict(), sigma_old=0.3)
    ref, _ = check_loss_bwd(gh, wl, dict(), sigma_old=0.3, kl_coef=0.04, expect_clip=True)
    assert ref["loss"] > ref0["loss"] and (ref["g"] != 0).sum() > (ref0["g"] != 0).sum()
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, use_oracle_lse=False, kl_coef=0.04)   # one-call route, penalty alone
    check_loss_bwd(gh, wl, dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=False, kl_coef=0.04,
                   entropy_coef=1e-3, grad_scale=4.0, stats=True)


def test_kl_penalty_needs_the_reference_logprobs(gh):
    wl = ai.make_config("cfg1")
    d = gh.logits_to_dev(wl.logits_rows(0, wl.T), wl.dtype)
    with pytest.raises(Exception):
        gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, wl.targets, None, np.zeros(wl.T), wl.token_rollout,
                        np.zeros(wl.R), np.zeros(wl.R), kl_coef=0.1)


def test_entropy_bonus_needs_the_entropy_array(gh):
    wl = ai.make_config("cfg1")
    d = gh.logits_to_dev(wl.logits_rows(0, wl.T), wl.dtype)
    lse = torch.zeros(wl.T, device=gh.DEV)
    with pytest.raises(Exception):
        gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, wl.targets, lse, np.zeros(wl.T), wl.token_rollout,
                        np.zeros(wl.R), np.zeros(wl.R), entropy_coef=1e-3)


# V >= 8192 with aligned rows takes the single-pass kernel when lse is not given: 151936 and
# 163840 (its largest row) use 20 vectors per thread, 32768 and 8200 (ragged tail) use 8;
# 163848 is one vector too long and falls back to forward + gradient passes, as do the others
# (262144: the largest vocabularies in use).
@pytest.mark.parametrize("V,ld,slots", [(151936, 151936, 6), (4999, 4999, 10), (1000, 1008, 10), (32768, 32768, 10),
                                        (8200, 8200, 10), (163840, 163848, 4), (163848, 163848, 4),
                                        (262144, 262144, 4)])
def test_loss_bwd_cfg2_reduced(gh, V, ld, slots):
    wl = ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots)
    check_loss_bwd(gh, wl, dict())
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, use_oracle_lse=False, expect_clip=True)
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, use_oracle_lse=False, stats=True)
    check_loss_bwd(gh, wl, dict(), inplace=True)
    check_loss_bwd(gh, wl, dict(), inplace=True, use_oracle_lse=False, stats=True, grad_scale=3.0)


@pytest.mark.parametrize("V,ld,slots", [(151936, 151936, 6), (4999, 4999, 10), (1000, 1008, 10), (32768, 32768, 8)])
def test_loss_bwd_f16(gh, V, ld, slots):
    """fp16 logits and gradients.  grad_scale lifts the gradient entries out of fp16's subnormal
    range, as a caller training in fp16 would; the unscaled run checks the rounding to that grid."""
    def wl():
        return ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots, dtype="f16")
    check_loss_bwd(gh, wl(), dict(), grad_scale=4096.0)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, expect_clip=True, grad_scale=4096.0, stats=True)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, inplace=True, grad_scale=4096.0)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3)
    check_loss_bwd(gh, wl(), dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=False,
                   entropy_coef=1e-3, kl_coef=0.04, grad_scale=4096.0)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, adv_map=lambda a: np.abs(a) + np.float32(0.25), strict_loss=True)


@pytest.mark.parametrize("V,ld,slots", [(151936, 151936, 6), (4999, 5008, 10), (1000, 1003, 10), (32768, 32768, 8)])
def test_loss_bwd_f8(gh, V, ld, slots):
    """8-bit float logits and gradients.  The gradient entries are far below the format's grid (2^-9), so a
    grad_scale lifts them (512: the largest entries of these short-response batches stay below the format's
    maximum of 448); the unscaled run checks that everything rounds to that grid (mostly to zero)."""
    def wl():
        return ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots, dtype="f8e4m3")
    check_loss_bwd(gh, wl(), dict(), grad_scale=512.0)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, expect_clip=True, grad_scale=512.0, stats=True)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, inplace=True, grad_scale=512.0,
                   untouched="half")
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3)
    check_loss_bwd(gh, wl(), dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=False,
                   entropy_coef=1e-3, kl_coef=0.04, grad_scale=512.0)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, adv_map=lambda a: np.abs(a) + np.float32(0.25), strict_loss=True)


def test_f8_gradient_rounding_bit_exact(gh):
    """The narrowing of gradient entries to the 8-bit float, bit for bit.  Rows [0, -384] with lse = 0 and the
    second token sampled have p = (1, 0) exactly, so with weight 1, ratio 1 and advantage -x the stored entry of
    the sampled token is x itself: every representable value, every midpoint of two neighbours (ties to even),
    values around the subnormal grid, and magnitudes beyond 448 (saturate) are compared with the host rounding
    (itself pinned against torch)."""
    grid = orc.widen(np.arange(127, dtype=np.uint8), "f8e4m3")
    mid = (grid[:-1] + grid[1:]) / 2
    rng = np.random.default_rng(5)
    x = np.concatenate([grid, mid, np.nextafter(mid.astype(np.float32), np.float32(0)),
                        np.nextafter(mid.astype(np.float32), np.float32(1e9)),
                        np.abs(rng.standard_normal(2000)) * 30, np.abs(rng.standard_normal(500)) * 0.01,
                        [449.0, 463.9, 464.0, 479.9, 480.0, 1e4, 3e38, 2.0 ** -10, 2.0 ** -11, 1e-30]]).astype(np.float32)
    x = np.concatenate([x, -x])
    x = x[x != 0]                       # advantage 0 switches the row off
    T = len(x)
    want = ai.f32_to_f8e4m3_bits(x)
    for V in (2, 16):                   # 2: rows of 2 bytes, element-wise stores; 16: one 16-byte vector per row
        z = np.tile(ai.f32_to_f8e4m3_bits(np.float32([0.0] + [-384.0] * (V - 1))), (T, 1))
        targets = np.ones(T, np.int32)
        lse = np.zeros(T, np.float32)
        old = np.full(T, -384.0, np.float32)          # = the current log-prob: ratio exactly 1, never clipped
        out = gh.run_loss_bwd(gh.logits_to_dev(z, "f8e4m3"), T, V, V, targets, gh.dev(lse), old,
                              np.arange(T, dtype=np.int32), -x.astype(np.float64), np.ones(T), eps=0.2)
        assert out["err"] == 0
        got = gh.raw_bits(out["dlogits"]).cpu().numpy()
        assert np.array_equal(got[:, 1], want)            # g (1 - p_1) = x
        assert np.array_equal(got[:, 0], want ^ 0x80)     # g (0 - p_0) = -x
        assert not (got[:, 2:] & 0x7F).any()              # -x * 0: a zero of either sign


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_all_storage_types(gh, seed):
    """Seeded random vocabulary sizes, row pitches (aligned and not), batch shapes, storage types and call
    variants: statistics, loss and gradient against the checker as in the fixed cases."""
    rng = np.random.default_rng(2000 + seed)
    dtype = ["bf16", "f32", "f16", "f8e4m3"][seed % 4]
    V = int(rng.choice([rng.integers(1, 64), rng.integers(64, 3000), rng.integers(3000, 40000)]))
    ld = V + int(rng.choice([0, 0, rng.integers(1, 40)]))
    slots = int(rng.integers(3, 13))

    def wl():
        return ai.make_config("cfg2", seed=100 + seed, V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots - 1, dtype=dtype)
    active = (wl().token_rollout >= 0).astype(np.uint8)
    assert check_fwd(gh, wl()) == 0
    assert check_fwd(gh, wl(), row_active=active, offset_elems=int(rng.integers(0, 9))) == 0
    gs = {"f16": 4096.0, "f8e4m3": 256.0}.get(dtype, float(rng.choice([1.0, 3.0])))
    for _ in range(3):
        terms = rng.random() < 0.4
        check_loss_bwd(gh, wl(), dict(reject_enable=int(rng.integers(2)), posterior_mode=int(rng.integers(2))),
                       sigma_old=float(rng.choice([0.05, 0.3])), use_oracle_lse=bool(rng.integers(2)),
                       inplace=bool(rng.integers(2)), grad_scale=gs, stats=False,
                       entropy_coef=0.01 if terms else 0.0, kl_coef=0.04 if terms and rng.random() < 0.5 else 0.0,
                       untouched=[None, "half", "all"][int(rng.integers(3))])


def test_loss_bwd_cfg3_reduced(gh):
    wl = ai.make_config("cfg3", V=151936, T=320, Q=64, len_lo=1, len_hi=12)
    ref, _ = check_loss_bwd(gh, wl, dict())
    assert (ref["g"] == 0).any() and (ref["g"] != 0).any()
    wl = ai.make_config("cfg3", V=151936, T=320, Q=64, len_lo=1, len_hi=12)
    check_loss_bwd(gh, wl, dict(), sigma_old=0.3, use_oracle_lse=False, stats=True)
    check_loss_bwd(gh, wl, dict(reject_enable=1), sigma_old=0.3, use_oracle_lse=False)
    wl = ai.make_config("cfg3", V=8000, T=700, Q=64, len_lo=1, len_hi=12)
    check_loss_bwd(gh, wl, dict(reject_enable=1), sigma_old=0.3, use_oracle_lse=False, expect_clip=True)
    check_loss_bwd(gh, wl, dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, expect_clip=True)


def test_streaming_kernel_optional_terms_several_rows_per_workgroup(gh):
    """V = 151936 with 320 rows: more rows than compute units, so the persistent workgroups of the
    streaming single-pass kernel refill their slots with a second row and draw it from the row
    counter, here in the variant that carries the optional terms (entropy bonus, Table 8; KL
    penalty, Eq. 2's beta term) and with the gradient written over the logits."""
    def wl():
        return ai.make_config("cfg3", V=151936, T=320, Q=64, len_lo=1, len_hi=12)
    ref, _ = check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, entropy_coef=0.02, expect_clip=True)
    assert ((ref["g"] == 0) & (ref["e"] != 0)).any()
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, kl_coef=0.04, stats=True)
    ref, _ = check_loss_bwd(gh, wl(), dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=False,
                            kl_coef=0.04, entropy_coef=1e-3, inplace=True, grad_scale=4.0)
    assert (ref["e"] == 0).any() and (ref["e"] != 0).any()      # dropped rollouts: rows with neither term
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, inplace=True)      # plain variant, in place
    check_loss_bwd(gh, wl(), dict(reject_enable=1), use_oracle_lse=False, inplace=True, stats=True)


# 151936 with 384 rows: the streaming kernel with several rows per workgroup; 32768: one workgroup per row;
# 4999 / 1000: the forward + gradient route (row kernels); with the checker's lse: the gradient kernels alone
# (151936: one vector per thread in segments).
@pytest.mark.parametrize("V,ld,slots,dtype", [(151936, 151936, 24, "bf16"), (32768, 32768, 10, "bf16"),
                                              (4999, 4999, 10, "bf16"), (1000, 1008, 10, "f32"),
                                              (151936, 151936, 6, "f16")])
def test_untouched_padding_rows(gh, V, ld, slots, dtype):
    """Padding rows marked AERO_ROW_UNTOUCHED: no gradient row is written for them (the buffer keeps its
    contents), their scalar outputs are 0, and every other row - plain padding included - is as before."""
    def wl():
        return ai.make_config("cfg2", V=V, ld=ld, slots=slots, len_lo=1, len_hi=slots - 1, dtype=dtype)
    gs = 4096.0 if dtype == "f16" else 1.0
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, untouched="half", grad_scale=gs)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, untouched="all", stats=True, grad_scale=gs)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=True, untouched="half", grad_scale=gs)
    check_loss_bwd(gh, wl(), dict(), sigma_old=0.3, use_oracle_lse=False, untouched="half", inplace=True, grad_scale=gs)
    check_loss_bwd(gh, wl(), dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=False,
                   untouched="all", entropy_coef=1e-3, kl_coef=0.04, grad_scale=gs)


# Well-conditioned losses: every term carries one sign, so nothing cancels and the stated
# tolerance (1e-4 relative) is enforced with no rounding floor.
@pytest.mark.parametrize("cfg,kw", [("cfg1", dict()),
                                    ("cfg2", dict(V=151936, ld=151936, slots=6, len_lo=1, len_hi=6)),
                                    ("cfg3", dict(V=151936, T=320, Q=64, len_lo=1, len_hi=12)),
                                    ("cfg2", dict(V=4999, ld=4999, slots=10, len_lo=1, len_hi=10))])
def test_loss_strict_tolerance_one_sign_advantages(gh, cfg, kw):
    for route in (True, False):   # statistics given / computed in the call (single pass where it applies)
        check_loss_bwd(gh, ai.make_config(cfg, **kw), dict(), sigma_old=0.3, use_oracle_lse=route, expect_clip=True,
                       adv_map=lambda a: np.abs(a) + np.float32(0.25), strict_loss=True)
        check_loss_bwd(gh, ai.make_config(cfg, **kw), dict(), sigma_old=0.05, use_oracle_lse=route,
                       adv_map=lambda a: -np.abs(a) - np.float32(0.25), strict_loss=True)


@pytest.mark.parametrize("cfg,kw", [("cfg1", dict()), ("cfg3", dict(V=151936, T=320, Q=64, len_lo=1, len_hi=12))])
def test_loss_strict_tolerance_posterior_mode(gh, cfg, kw):
    """Every group all-wrong: in posterior mode (Strategy 2) each kept rollout gets the same negative
    advantage (-1/3 at n = 8 with the uniform prior), the loss is a sum of one-signed terms."""
    for route in (True, False):
        wl = ai.make_config(cfg, **kw)
        wl.rewards[:] = 0.0
        ref, _ = check_loss_bwd(gh, wl, dict(reject_enable=1, posterior_mode=1), sigma_old=0.3, use_oracle_lse=route,
                                expect_clip=True, strict_loss=True)
        assert (ref["g"] != 0).any() and ref["loss"] > 0


def test_loss_is_run_to_run_identical_and_loss_only_mode(gh):
    wl = ai.make_config("cfg3", V=8000, T=3000, Q=64, len_lo=1, len_hi=40)
    host = wl.logits_rows(0, wl.T)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
    lp_ref, _, lse_ref = orc.logprob_fwd(host, wl.dtype, wl.V, wl.targets)
    old = ai.draw_old_logprob(lp_ref, 5, sigma=0.2)
    d = gh.logits_to_dev(host, wl.dtype)
    outs = [gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, wl.targets, None, old, wl.token_rollout, ga["adv"], ga["weight"],
                            want_dlogits=(k < 2)) for k in range(3)]
    assert outs[0]["loss"].view(torch.int32).item() == outs[1]["loss"].view(torch.int32).item()
    assert outs[0]["loss"].view(torch.int32).item() == outs[2]["loss"].view(torch.int32).item()
    assert torch.equal(outs[0]["dlogits"].view(torch.int16), outs[1]["dlogits"].view(torch.int16))


def test_bad_rollout_index_and_empty_batch(gh):
    wl = ai.make_config("cfg2", V=512, slots=4, len_lo=4, len_hi=4)
    host = wl.logits_rows(0, wl.T)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
    tr = wl.token_rollout.copy()
    tr[3] = wl.R + 5
    d = gh.logits_to_dev(host, wl.dtype)
    out = gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, wl.targets, None, np.zeros(wl.T, np.float32) - 6.0, tr,
                          ga["adv"], ga["weight"])
    assert out["err"] & 4 and not out["dlogits"][3].float().any()
    out = gh.run_loss_bwd(d[:0], 0, wl.V, wl.ld, np.zeros(0, np.int32), None, np.zeros(0, np.float32),
                          np.zeros(0, np.int32), ga["adv"], ga["weight"])
    assert out["loss"].item() == 0.0 and out["clip_frac"].item() == 0.0


def test_raw_c_abi_call_without_the_binding(gh):
    """aero_logprob_fwd called through ctypes directly: plain device addresses and sizes, the NULL
    (default) stream, status code returned; results against the checker."""
    import ctypes as C
    from paper_2602_14338_amd import binding
    lib = C.CDLL(binding.library_path())
    p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.aero_logprob_fwd.restype = i32
    lib.aero_logprob_fwd.argtypes = [p, i32, i64, i32, i64, p, p, p, p, p, p, p]
    wl = ai.make_config("cfg2", V=4999, ld=5008, slots=5, len_lo=1, len_hi=5)
    host = wl.logits_rows(0, wl.T)
    ref = orc.logprob_fwd(host, "bf16", wl.V, wl.targets)
    z = gh.logits_to_dev(host, "bf16")
    tg = gh.dev(wl.targets)
    lp, ent, lse = (torch.full((wl.T,), 7.0, device=gh.DEV) for _ in range(3))
    torch.cuda.synchronize()
    st = lib.aero_logprob_fwd(z.data_ptr(), 1, wl.T, wl.V, wl.ld, tg.data_ptr(), None, lp.data_ptr(), ent.data_ptr(),
                              lse.data_ptr(), None, None)
    assert st == 0
    torch.cuda.synchronize()
    for got, want in ((lp, ref[0]), (ent, ref[1]), (lse, ref[2])):
        assert np.abs(got.cpu().numpy().astype(np.float64) - want).max() <= LP_TOL
    assert lib.aero_logprob_fwd(z.data_ptr(), 1, wl.T, wl.V, wl.V - 1, tg.data_ptr(), None, lp.data_ptr(), None,
                                lse.data_ptr(), None, None) == 2      # AERO_ERR_SHAPE: ld < V
    assert lib.aero_logprob_fwd(z.data_ptr(), 5, wl.T, wl.V, wl.ld, tg.data_ptr(), None, lp.data_ptr(), None,
                                lse.data_ptr(), None, None) == 3      # AERO_ERR_DTYPE


def test_ignored_rows_are_not_flagged(gh):
    """Padding rows (rollout index -1) and rows switched off with row_active may hold anything in
    their other fields, e.g. a sampled-token id past the vocabulary: no error bit, zero outputs.
    Covers the forward call, the two-call loss route, and both single-pass kernels."""
    for V, slots in ((512, 6), (32768, 6), (151936, 4)):
        wl = ai.make_config("cfg2", V=V, slots=slots, len_lo=1, len_hi=slots - 1)
        host = wl.logits_rows(0, wl.T)
        pad = wl.token_rollout < 0
        assert pad.any()
        tg = wl.targets.copy()
        tg[pad] = V + 7
        ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
        d = gh.logits_to_dev(host, wl.dtype)
        lp, ent, lse, err = gh.run_fwd(d, wl.T, wl.V, wl.ld, tg, (~pad).astype(np.uint8))
        assert err == 0 and not lp[torch.from_numpy(pad).to(gh.DEV)].any()
        _, _, _, err = gh.run_fwd(d, wl.T, wl.V, wl.ld, tg, None)      # not switched off: flagged
        assert err == 2
        old = np.full(wl.T, -12.0, np.float32)
        for lse_arg in (lse, None):
            out = gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, tg, lse_arg, old, wl.token_rollout, ga["adv"], ga["weight"])
            assert out["err"] == 0
            assert not out["dlogits"][torch.from_numpy(pad).to(gh.DEV)].float().any()
        tr = wl.token_rollout.copy()
        tr[~pad] = np.where(np.arange((~pad).sum()) % 3 == 0, wl.R + 1, tr[~pad])   # real bad indices are flagged
        out = gh.run_loss_bwd(d, wl.T, wl.V, wl.ld, tg, None, old, tr, ga["adv"], ga["weight"])
        assert out["err"] == 4


def test_host_side_argument_errors(gh):
    import paper_2602_14338_amd as aero
    z = torch.zeros((4, 16), dtype=torch.bfloat16, device=gh.DEV)
    t = torch.zeros(4, dtype=torch.int32, device=gh.DEV)
    f = torch.zeros(4, device=gh.DEV)
    with pytest.raises(aero.AeroError, match="leading dimension"):
        aero.aero_logprob_fwd(z, 4, 16, 8, t, None, f, f, f)
    with pytest.raises(aero.AeroError, match="leading dimension"):
        aero.aero_logprob_fwd(z, 4, 0, 16, t, None, f, f, f)
    with pytest.raises(aero.AeroError, match="NULL"):
        aero.aero_logprob_fwd(z, 4, 16, 16, None, None, f, f, f)
    with pytest.raises(aero.AeroError, match="unsupported dtype"):
        aero.aero_logprob_fwd(z.to(torch.float64), 4, 16, 16, t, None, f, f, f)
    with pytest.raises(aero.AeroError, match="workspace"):
        aero.aero_grpo_loss_bwd(z, 4, 16, 16, t, None, f, t, f, f, 4, 0.2, 0.2, 1.0, f[:1], None, None, None,
                                torch.zeros(8, dtype=torch.uint8, device=gh.DEV))
