"""Pins for the float64 checker: what the paper and the mathematics fix, never the checker
itself.  Closed forms come from the proof of Theorem 4.1 / Lemma 4.2, library routines
(statistics.pstdev, scipy.special.log_softmax / logsumexp, scipy.stats.entropy, torch
autograd in float64) serve as independent routes to the same definitions, and central
finite differences pin every gradient."""
import itertools
import math
import os
import statistics

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

import aero_inputs as ai
from oracle import aero_oracle as orc
from oracle.aero_oracle import AdvParams

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def paper_values():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = [s.strip() for s in line.split("=")]
            out[k] = float(v)
    return out


PV = paper_values()


def one_group(rewards, lengths=None, keys=None, **kw):
    r = np.asarray(rewards, np.float32)
    L = np.full(len(r), 7, np.int32) if lengths is None else np.asarray(lengths, np.int32)
    off = np.array([0, len(r)], np.int32)
    return orc.group_advantage(r, L, off, keys, AdvParams(**kw))


# ------------------------------------------------------------------ storage formats

def test_bf16_roundtrip_matches_torch():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(100000) * 3).astype(np.float32)
    x[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38]   # ties and near-overflow
    bits = ai.f32_to_bf16_bits(x)
    tb = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, tb.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(orc.widen(bits, "bf16"), tb.double().numpy())


def test_f16_roundtrip_matches_torch():
    """binary16 storage: the generator's rounding and the checker's widening against torch's
    conversions, bit for bit (ties, subnormals, the largest finite value, every bit pattern)."""
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100000) * 3).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, 1.00048828125, 1.00146484375, 65504.0, 5.9604645e-8, 3.0e-8]
    bits = ai.f32_to_f16_bits(x)
    th = torch.from_numpy(x).to(torch.float16)
    assert np.array_equal(bits, th.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(orc.widen(bits, "f16"), th.double().numpy())
    every = np.arange(65536, dtype=np.uint16)
    finite = (every & 0x7C00) != 0x7C00
    want = torch.from_numpy(every.view(np.int16)).view(torch.float16).double().numpy()
    assert np.array_equal(orc.widen(every, "f16")[finite], want[finite])
    assert orc.widen(np.array([0x3C00, 0xC000, 0x0001, 0x7BFF], np.uint16), "f16").tolist() == \
        [1.0, -2.0, 2.0 ** -24, 65504.0]


def test_f8e4m3_roundtrip_matches_torch():
    """8-bit float storage (4 exponent, 3 mantissa bits, no infinities): the checker's widening of all
    256 patterns and the generator's rounding against torch's conversions, bit for bit; the values
    the format is defined by (largest 448, smallest subnormal 2^-9, one NaN per sign); ties go to the
    even mantissa, also across a power of two and into the subnormals."""
    every = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(every).view(torch.float8_e4m3fn).float().double().numpy()
    got = orc.widen(every, "f8e4m3")
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.isnan(got).sum() == 2
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert orc.widen(np.array([0x7E, 0x01, 0x38, 0xC0, 0x08, 0x00, 0x80], np.uint8), "f8e4m3").tolist() == \
        [448.0, 2.0 ** -9, 1.0, -2.0, 2.0 ** -6, 0.0, -0.0]
    assert np.all(np.diff(got[:127]) > 0)                     # codes 0..126 ascend in value
    rng = np.random.default_rng(3)
    x = np.concatenate([(rng.standard_normal(200000) * 3).astype(np.float32),
                        (rng.standard_normal(20000) * 0.01).astype(np.float32)])
    mid = ((got[:126] + got[1:127]) / 2).astype(np.float32)   # every midpoint of two neighbours is a float32
    x = np.concatenate([x, mid, -mid, got[:127].astype(np.float32), np.float32([440.0, 447.9, 448.0, -448.0])])
    bits = ai.f32_to_f8e4m3_bits(x)
    tb = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(bits, tb)
    assert ai.f32_to_f8e4m3_bits(np.float32([1.0625, 1.1875, 0.0009765625, 1000.0, -1000.0])).tolist() == \
        [0x38, 0x3A, 0x00, 0x7E, 0xFE]                        # ties to even; 2^-10 -> 0; beyond the range -> 448


# ------------------------------------------------------------------ group statistics

@pytest.mark.parametrize("n", range(2, 17))
def test_advantage_closed_forms(n):
    """Theorem 4.1's proof: a+ = (1-mu)/sigma = sqrt(m/c), a- = -mu/sigma = -sqrt(c/m)."""
    for c in range(1, n):
        m = n - c
        r = [1.0] * c + [0.0] * m
        out = one_group(r)
        a = out["adv"]
        assert np.allclose(a[:c], math.sqrt(m / c), rtol=1e-14)
        assert np.allclose(a[c:], -math.sqrt(c / m), rtol=1e-14)
        assert abs(a.sum()) < 1e-12 and abs((a * a).sum() - n) < 1e-12
        assert out["zero_var"][0] == 0 and out["keep_mask"].all()
        # balance term of Lemma 4.2 is the variance and never exceeds 1/4
        var = c * m / (c + m) ** 2
        assert var <= PV["balance_term_max"] and (var == PV["balance_term_max"]) == (m == c)


def test_advantage_matches_library_pstdev_all_patterns():
    for n in range(1, 9):
        for pat in itertools.product([0.0, 1.0], repeat=n):
            a = one_group(pat)["adv"]
            sd = statistics.pstdev(pat)
            mu = statistics.fmean(pat)
            want = [0.0] * n if sd == 0 else [(x - mu) / sd for x in pat]
            assert np.allclose(a, want, rtol=1e-13, atol=0)


def test_general_rewards_plain_mode():
    rng = np.random.default_rng(3)
    r = rng.normal(size=11).astype(np.float32)
    out = one_group(r)
    r64 = r.astype(np.float64)
    assert np.allclose(out["adv"], (r64 - r64.mean()) / np.std(r64), rtol=1e-13)
    assert out["err"] == 0
    assert one_group(r, reject_enable=1)["err"] & orc.ERR_NONBINARY_REWARD


def test_all_equal_groups_give_zero():
    """Sec. 3.2: all-fail (and all-correct) groups have zero advantage."""
    for n in (1, 2, 8, 16):
        for v in (0.0, 1.0):
            out = one_group([v] * n)
            assert not out["adv"].any() and out["zero_var"][0] == 1
            out = one_group([v] * n, reject_enable=1)
            assert not out["adv"].any() and not out["keep_mask"].any() and not out["weight"].any()
            assert out["kept_offsets"].tolist() == [0, 0] and len(out["kept_index"]) == 0


def test_rescued_pair_is_plus_minus_one():
    out = one_group([0.0, 1.0], reject_enable=1)
    assert int(PV["rescued_group_size"]) == 2
    assert out["adv"].tolist() == [-1.0, 1.0]


def test_categories_follow_the_case_formula():
    n = int(PV["n_explore"])
    for c in range(n + 1):
        u = c / n
        want = (orc.CAT_ZERO if u == 0 else orc.CAT_PARTIAL if u < PV["tau"]
                else orc.CAT_GOOD if u < 1 else orc.CAT_PERFECT)
        out = one_group([1.0] * c + [0.0] * (n - c), reject_enable=1)
        assert out["category"][0] & 3 == want
        assert bool(out["category"][0] & orc.CAT_RESCUE_BIT) == (c <= PV["rescue_S"])
    # rescue threshold S = 2 marks c <= 2 without changing the four-way category
    out = one_group([1, 1, 0, 0, 0, 0, 0, 0], s_rescue=2)
    assert out["category"][0] == orc.CAT_PARTIAL | orc.CAT_RESCUE_BIT
    # odd n: 2c < n is partial (u < 1/2)
    assert one_group([1, 1, 0, 0, 0])["category"][0] & 3 == orc.CAT_PARTIAL
    assert one_group([1, 1, 1, 0, 0])["category"][0] & 3 == orc.CAT_GOOD


def test_high_success_example_is_kept_whole():
    """App. B.3.4's example group (8 rollouts, 5 correct) is in the stratum AERO keeps whole."""
    n, c = int(PV["example_high_success_n"]), int(PV["example_high_success_c"])
    out = one_group([1.0] * c + [0.0] * (n - c), reject_enable=1)
    assert out["category"][0] & 3 == orc.CAT_GOOD and out["keep_mask"].sum() == n


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_rejection_counts_and_balance(k):
    """Strategy 3: all c correct rollouts + m = k c incorrect ones (capped by what exists)."""
    for n in range(3, 17):
        for c in range(1, n):
            if 2 * c >= n:
                continue
            out = one_group([0.0] * (n - c) + [1.0] * c, reject_enable=1, k_ratio=k)
            m = min(k * c, n - c)
            keep = out["keep_mask"]
            assert keep[n - c:].all() and keep[:n - c].sum() == m and keep[:m].all()
            a = out["adv"][keep == 1]
            assert abs(a.sum()) < 1e-12 and abs((a * a).sum() - (c + m)) < 1e-12
            if k == 1:   # balanced subset: advantages are exactly +-1 (Lemma 4.2, k = 1)
                assert sorted(set(a.tolist())) == [-1.0, 1.0]
            assert not out["adv"][keep == 0].any() and not out["weight"][keep == 0].any()


def test_keep_set_matches_rank_counting_brute_force():
    """Which incorrect rollouts survive: those with fewer than m incorrect rollouts ahead
    of them in (key, index) order.  All reward patterns up to n = 9, keys with many ties."""
    rng = np.random.default_rng(11)
    for n in range(2, 10):
        for pat in itertools.product([0.0, 1.0], repeat=n):
            keys = rng.integers(0, 4, size=n).astype(np.uint32)
            c = int(sum(pat))
            out = one_group(pat, keys=keys, reject_enable=1, k_ratio=1)
            want = np.zeros(n, np.uint8)
            if 0 < c and 2 * c < n:
                m = min(c, n - c)
                for i in range(n):
                    if pat[i] == 1.0:
                        want[i] = 1
                    else:
                        ahead = sum(1 for j in range(n) if pat[j] == 0.0 and
                                    (keys[j], j) < (keys[i], i))
                        want[i] = ahead < m
            elif 0 < c < n:
                want[:] = 1
            assert np.array_equal(out["keep_mask"], want)
            assert np.array_equal(out["kept_index"], np.nonzero(want)[0])


def test_posterior_mode():
    """Strategy 2: u~ = (c + 1)/(n + 2) stays inside (0, 1); 4 rollouts are kept.  The
    divisor sqrt(u~(1-u~)) is a reading taken here, so the +-1/3 below pins the reading's
    closed form only."""
    n = int(PV["n_explore"])
    a0, b0 = PV["prior_alpha0"], PV["prior_beta0"]
    keys = np.array([5, 1, 7, 1, 9, 0, 3, 2], np.uint32)
    for v, u_want in ((0.0, 0.1), (1.0, 0.9)):
        out = one_group([v] * n, keys=keys, reject_enable=1, posterior_mode=1, alpha0=a0, beta0=b0)
        assert out["keep_mask"].sum() == PV["zero_adv_kept"]
        assert out["kept_index"].tolist() == [1, 3, 5, 7]          # keys 1, 1, 0, 2
        u = (v * n + a0) / (n + a0 + b0)
        assert abs(u - u_want) < 1e-15 and 0 < u < 1
        kept = out["adv"][out["keep_mask"] == 1]
        assert np.allclose(kept, (v - u) / math.sqrt(u * (1 - u)), rtol=1e-14)
        assert np.allclose(kept, -1 / 3 if v == 0 else 1 / 3, rtol=1e-14)
        assert out["zero_var"][0] == 1 and (out["weight"][out["keep_mask"] == 1] > 0).all()
    # a group smaller than 4 keeps what it has
    assert one_group([0, 0, 0], reject_enable=1, posterior_mode=1)["keep_mask"].sum() == 3
    # mixed groups are untouched by posterior mode
    a = one_group([1, 0, 0, 1], posterior_mode=1)["adv"]
    assert a.tolist() == [1.0, -1.0, -1.0, 1.0]


def test_weights_and_csr_on_ragged_batch():
    wl = ai.make_config("cfg3", Q=40)
    for kw in (dict(), dict(reject_enable=1), dict(reject_enable=1, posterior_mode=1)):
        out = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams(**kw))
        off = wl.group_offsets
        groups_with_kept = 0
        for q in range(wl.Q):
            sl = slice(off[q], off[q + 1])
            k = out["keep_mask"][sl]
            assert out["kept_offsets"][q + 1] - out["kept_offsets"][q] == k.sum()
            if k.sum():
                groups_with_kept += 1
                # Eq. 2: within a group the sequence means are averaged with weight 1/N
                wl_sum = (out["weight"][sl] * wl.lengths[sl])[k == 1]
                assert np.allclose(wl_sum, 1.0 / (wl.Q * k.sum()), rtol=1e-14)
        assert abs((out["weight"] * wl.lengths).sum() - groups_with_kept / wl.Q) < 1e-12
        ki = out["kept_index"]
        assert np.all(np.diff(ki) > 0) and np.array_equal(ki, np.nonzero(out["keep_mask"])[0])
        assert out["kept_offsets"][-1] == len(ki)


def test_empty_group_and_empty_batch():
    out = orc.group_advantage(np.array([1, 0], np.float32), np.array([3, 3], np.int32),
                              np.array([0, 0, 2, 2], np.int32), None, AdvParams(reject_enable=1))
    assert out["category"].tolist() == [orc.CAT_ZERO | orc.CAT_RESCUE_BIT, orc.CAT_GOOD,
                                        orc.CAT_ZERO | orc.CAT_RESCUE_BIT]
    assert out["zero_var"].tolist() == [1, 0, 1] and out["kept_offsets"].tolist() == [0, 0, 2, 2]
    out = orc.group_advantage(np.zeros(0, np.float32), np.zeros(0, np.int32), np.array([0], np.int32),
                              None, AdvParams())
    assert len(out["adv"]) == 0 and out["kept_offsets"].tolist() == [0]


# ------------------------------------------------------------------ softmax statistics

def test_logprob_against_scipy():
    rng = np.random.default_rng(5)
    for V, sigma in ((7, 1.0), (1000, 3.0), (151936, 3.0)):
        z = rng.normal(0, sigma, size=V)
        y = int(rng.integers(V))
        lp, ent, lse = orc.logprob_row(z, y)
        assert abs(lse - scipy.special.logsumexp(z)) < 1e-12
        assert abs(lp - scipy.special.log_softmax(z)[y]) < 1e-12
        assert abs(ent - scipy.stats.entropy(scipy.special.softmax(z))) < 1e-11
        assert abs(np.exp(z - lse).sum() - 1.0) < 1e-12


def test_logprob_special_cases():
    V = 1187
    lp, ent, lse = orc.logprob_row(np.full(V, 2.5), 17)
    assert abs(lp + math.log(V)) < 1e-13 and abs(ent - math.log(V)) < 1e-12
    z = np.full(V, -40.0)
    z[3] = 40.0
    lp, ent, lse = orc.logprob_row(z, 3)
    assert abs(lp) < 1e-30 + 1e-12 and abs(ent) < 1e-12
    rng = np.random.default_rng(6)
    z = rng.normal(0, 3, size=V)
    a = orc.logprob_row(z, 5)
    b = orc.logprob_row(z + 1234.5, 5)
    assert abs(a[0] - b[0]) < 1e-10 and abs(a[1] - b[1]) < 1e-10 and abs(b[2] - a[2] - 1234.5) < 1e-10
    # large logits must not overflow
    assert np.isfinite(orc.logprob_row(z * 1e3, 5)).all()


def test_logprob_against_long_double_two_pass():
    rng = np.random.default_rng(7)
    z = rng.normal(0, 3, size=300)
    zl = z.astype(np.longdouble)
    tot = np.longdouble(0)
    for v in zl:
        tot += np.exp(v)
    lse = np.log(tot)
    p = np.exp(zl - lse)
    ent = -(p * (zl - lse)).sum()
    got = orc.logprob_row(z, 42)
    assert abs(got[2] - float(lse)) < 1e-13 and abs(got[0] - float(zl[42] - lse)) < 1e-13
    assert abs(got[1] - float(ent)) < 1e-12


def test_logprob_fwd_rows_masks_and_padding_columns():
    wl = ai.make_config("cfg2", V=1000, slots=8, len_lo=2, len_hi=8, ld=1008)
    logits = wl.logits_rows(0, wl.T)
    active = (wl.token_rollout >= 0).astype(np.uint8)
    tg = wl.targets.copy()
    tg[0] = -1
    lp, ent, lse = orc.logprob_fwd(logits, "bf16", wl.V, tg, active)
    assert np.isfinite(lp).all() and np.isfinite(lse).all()       # +inf pad columns never read
    assert lp[0] == 0 and ent[0] == 0 and lse[0] == 0
    assert not lp[active == 0].any() and not lse[active == 0].any()
    t = int(np.nonzero(active)[0][1])
    z = torch.from_numpy(logits[t, :wl.V].view(np.int16)).view(torch.bfloat16).double()
    assert abs(lp[t] - torch.log_softmax(z, 0)[tg[t]].item()) < 1e-12


# ------------------------------------------------------------------ loss and gradient

def tiny_problem(seed, T=12, V=9, R=4, sigma_old=0.3):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 2, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    tr = rng.integers(0, R, size=T).astype(np.int32)
    adv = rng.normal(size=R)
    adv[0] = 0.0
    w = rng.uniform(0.01, 0.1, size=R)
    lp = np.array([orc.logprob_row(z[t], y[t])[0] for t in range(T)])
    old = ai.draw_old_logprob(lp, seed, sigma=sigma_old).astype(np.float64)
    return z, y, tr, adv, w, old


def torch_loss(z, y, tr, adv, w, old, eps_lo, eps_hi):
    """Eq. 2 written with torch ops in float64; autograd supplies the gradient."""
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(zt, dim=1).gather(1, torch.tensor(y, dtype=torch.int64)[:, None])[:, 0]
    rho = torch.exp(lp - torch.tensor(old))
    A = torch.tensor(adv)[torch.tensor(tr, dtype=torch.int64)]
    W = torch.tensor(w)[torch.tensor(tr, dtype=torch.int64)]
    s = torch.minimum(rho * A, torch.clamp(rho, 1 - eps_lo, 1 + eps_hi) * A)
    loss = -(W * s).sum()
    loss.backward()
    return loss.item(), zt.grad.numpy()


@pytest.mark.parametrize("seed", range(6))
def test_loss_and_gradient_match_autograd(seed):
    z, y, tr, adv, w, old = tiny_problem(seed)
    out = orc.grpo_loss_bwd(None, "f64", z.shape[1], y, old, tr, adv, w, 0.2, 0.2, z64=z)
    loss, grad = torch_loss(z, y, tr, adv, w, old, 0.2, 0.2)
    assert abs(out["loss"] - loss) < 1e-13
    assert np.allclose(out["dlogits"], grad, rtol=1e-11, atol=1e-15)


def test_gradient_matches_central_differences_and_all_clip_cases_occur():
    eps_lo, eps_hi = 0.2, 0.2
    seen = set()
    for seed in range(8):
        z, y, tr, adv, w, old = tiny_problem(100 + seed, T=8, V=6)
        V = z.shape[1]
        f = lambda zz: orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, eps_lo, eps_hi,
                                         want_dlogits=False, z64=zz)["loss"]
        out = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, eps_lo, eps_hi, grad_scale=1.0, z64=z)
        h = 1e-6
        fd = np.zeros_like(z)
        for t in range(z.shape[0]):
            for j in range(V):
                zp, zm = z.copy(), z.copy()
                zp[t, j] += h
                zm[t, j] -= h
                fd[t, j] = (f(zp) - f(zm)) / (2 * h)
        assert np.allclose(out["dlogits"], fd, atol=1e-8)
        assert np.abs(out["dlogits"].sum(axis=1)).max() < 1e-15     # each row sums to zero
        for t in range(z.shape[0]):
            A = adv[tr[t]]
            if A == 0:
                assert not out["dlogits"][t].any() and out["g"][t] == 0
                continue
            rho = math.exp(out["logprob"][t] - old[t])
            case = (A > 0, "hi" if rho > 1 + eps_hi else "lo" if rho < 1 - eps_lo else "in")
            seen.add(case)
            flows = case in ((True, "in"), (True, "lo"), (False, "in"), (False, "hi"))
            assert (out["g"][t] != 0) == flows
            if not flows:                      # App. A.1: clipped tokens contribute zero
                assert not out["dlogits"][t].any()
            else:                              # gradient of the ratio is rho * grad log pi
                assert abs(out["g"][t] + w[tr[t]] * A * rho) < 1e-15
    assert len(seen) == 6


# ------------------------------------------------------------------ entropy bonus (Table 8)

def torch_loss_with_entropy(z, y, tr, adv, w, old, eps_lo, eps_hi, c_ent):
    """Eq. 2 minus c * sum_t w_t H_t, H from torch's own softmax; autograd gives the gradient.
    Rollouts with weight 0 are outside both sums."""
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    logp = torch.log_softmax(zt, dim=1)
    lp = logp.gather(1, torch.tensor(y, dtype=torch.int64)[:, None])[:, 0]
    rho = torch.exp(lp - torch.tensor(old))
    A = torch.tensor(adv)[torch.tensor(tr, dtype=torch.int64)]
    W = torch.tensor(w)[torch.tensor(tr, dtype=torch.int64)]
    s = torch.minimum(rho * A, torch.clamp(rho, 1 - eps_lo, 1 + eps_hi) * A)
    H = torch.distributions.Categorical(logits=zt).entropy()
    loss = -(W * s).sum() - c_ent * (W * H).sum()
    loss.backward()
    return loss.item(), zt.grad.numpy()


@pytest.mark.parametrize("seed", range(4))
def test_entropy_bonus_matches_autograd(seed):
    z, y, tr, adv, w, old = tiny_problem(200 + seed)
    w[1] = 0.0                                    # a dropped rollout: no loss, no entropy term
    for c_ent, gs in ((1e-3, 1.0), (0.5, 4.0)):
        out = orc.grpo_loss_bwd(None, "f64", z.shape[1], y, old, tr, adv, w, 0.2, 0.2, grad_scale=gs, z64=z,
                                entropy_coef=c_ent)
        loss, grad = torch_loss_with_entropy(z, y, tr, adv, w, old, 0.2, 0.2, c_ent)
        assert abs(out["loss"] - loss) < 1e-13
        assert np.allclose(out["dlogits"], gs * grad, rtol=1e-10, atol=1e-15)
        assert not out["dlogits"][tr == 1].any()
        # rollout 0 has advantage 0: only the entropy term reaches its rows
        assert out["dlogits"][tr == 0].any() and not out["g"][tr == 0].any()
        assert np.abs(out["dlogits"].sum(axis=1)).max() < 1e-15     # rows still sum to zero


def test_entropy_gradient_closed_forms_and_central_differences():
    V = 7
    # uniform policy: H = ln V is the maximum, its gradient vanishes
    z = np.full(V, 0.3)
    _, ent, lse = orc.logprob_row(z, 0)
    assert abs(ent - math.log(V)) < 1e-15
    assert np.abs(orc.entropy_grad_row(z, lse, ent)).max() < 1e-16
    # two-point policy (p, 1-p): H = -p ln p - q ln q, dH/dz_0 = p q ln(q / p)
    for p in (0.1, 0.5, 0.9):
        z2 = np.array([math.log(p), math.log(1 - p)])
        _, ent2, lse2 = orc.logprob_row(z2, 0)
        g2 = orc.entropy_grad_row(z2, lse2, ent2)
        assert abs(g2[0] - p * (1 - p) * math.log((1 - p) / p)) < 1e-15 and abs(g2.sum()) < 1e-16
    rng = np.random.default_rng(5)
    z = rng.normal(0, 2, size=V)
    _, ent, lse = orc.logprob_row(z, 0)
    an = orc.entropy_grad_row(z, lse, ent)
    h = 1e-6
    for j in range(V):
        zp, zm = z.copy(), z.copy()
        zp[j] += h
        zm[j] -= h
        fd = (orc.logprob_row(zp, 0)[1] - orc.logprob_row(zm, 0)[1]) / (2 * h)
        assert abs(an[j] - fd) < 1e-9
    # through the whole loss: with rho = 1 and all advantages 0 the loss is - c sum_t w_t H_t
    T, R = 6, 2
    zz = rng.normal(0, 1.5, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    tr = (np.arange(T) % R).astype(np.int32)
    w = np.array([0.25, 0.125])
    lp = np.array([orc.logprob_row(zz[t], y[t])[0] for t in range(T)])
    out = orc.grpo_loss_bwd(None, "f64", V, y, lp, tr, np.zeros(R), w, 0.2, 0.2, z64=zz, entropy_coef=0.01)
    H = np.array([orc.logprob_row(zz[t], y[t])[1] for t in range(T)])
    assert abs(out["loss"] + 0.01 * (w[tr] * H).sum()) < 1e-16 and out["clip_frac"] == 0.0
    assert not orc.grpo_loss_bwd(None, "f64", V, y, lp, tr, np.zeros(R), w, 0.2, 0.2, z64=zz)["dlogits"].any()


# ------------------------------------------------------------------ KL penalty (Eq. 2, beta term)

@pytest.mark.parametrize("seed", range(4))
def test_kl_penalty_matches_autograd(seed):
    z, y, tr, adv, w, old = tiny_problem(300 + seed)
    w[1] = 0.0
    tr[0], tr[1] = 0, 1                            # rollout 0 has advantage 0, rollout 1 weight 0
    rng = np.random.default_rng(seed)
    ref_lp = old + rng.normal(0, 0.2, size=old.shape)
    beta = 0.04
    out = orc.grpo_loss_bwd(None, "f64", z.shape[1], y, old, tr, adv, w, 0.2, 0.2, grad_scale=2.0, z64=z,
                            kl_coef=beta, ref_logprob=ref_lp, entropy_coef=0.01)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(zt, dim=1).gather(1, torch.tensor(y, dtype=torch.int64)[:, None])[:, 0]
    rho = torch.exp(lp - torch.tensor(old))
    A = torch.tensor(adv)[torch.tensor(tr, dtype=torch.int64)]
    W = torch.tensor(w)[torch.tensor(tr, dtype=torch.int64)]
    s = torch.minimum(rho * A, torch.clamp(rho, 0.8, 1.2) * A)
    d = torch.tensor(ref_lp) - lp
    kl = torch.exp(d) - d - 1
    H = torch.distributions.Categorical(logits=zt).entropy()
    loss = -(W * s).sum() + beta * (W * kl).sum() - 0.01 * (W * H).sum()
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-13
    assert np.allclose(out["dlogits"], 2.0 * zt.grad.numpy(), rtol=1e-10, atol=1e-15)
    assert not out["dlogits"][tr == 1].any()
    assert out["g"][tr == 0].any()                # advantage 0, but the penalty still pulls towards pi_ref


def test_kl_penalty_closed_forms():
    # the estimator is >= 0, zero with zero slope where pi = pi_ref, and the penalty alone gives
    # g = grad_scale beta w (1 - pi_ref / pi)
    V, T = 5, 4
    rng = np.random.default_rng(9)
    z = rng.normal(size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    tr = np.zeros(T, np.int32)
    lp = np.array([orc.logprob_row(z[t], y[t])[0] for t in range(T)])
    same = orc.grpo_loss_bwd(None, "f64", V, y, lp, tr, np.zeros(1), np.array([0.5]), 0.2, 0.2, z64=z,
                             kl_coef=0.1, ref_logprob=lp)
    assert same["loss"] == 0.0 and not same["g"].any() and not same["dlogits"].any()
    ref_lp = lp + np.array([0.3, -0.2, 0.05, -1.0])
    out = orc.grpo_loss_bwd(None, "f64", V, y, lp, tr, np.zeros(1), np.array([0.5]), 0.2, 0.2, grad_scale=3.0,
                            z64=z, kl_coef=0.1, ref_logprob=ref_lp)
    d = ref_lp - lp
    assert (np.exp(d) - d - 1 > 0).all()
    assert abs(out["loss"] - 0.1 * 0.5 * (np.exp(d) - d - 1).sum()) < 1e-16
    assert np.allclose(out["g"], 3.0 * 0.1 * 0.5 * (1 - np.exp(d)), rtol=1e-14)
    h = 1e-6
    for t in range(T):
        for j in range(V):
            zp, zm = z.copy(), z.copy()
            zp[t, j] += h
            zm[t, j] -= h
            f = lambda zz: orc.grpo_loss_bwd(None, "f64", V, y, lp, tr, np.zeros(1), np.array([0.5]), 0.2, 0.2,
                                             want_dlogits=False, z64=zz, kl_coef=0.1, ref_logprob=ref_lp)["loss"]
            assert abs((f(zp) - f(zm)) / (2 * h) - out["dlogits"][t, j] / 3.0) < 1e-9


def test_clip_edge_counts_as_unclipped():
    for A, lp_minus_old in ((1.0, math.log(1.2)), (-1.0, math.log(0.8))):
        rho = math.exp(lp_minus_old)
        edge_hi, edge_lo = rho - 1.0, 1.0 - rho
        term, g, unclipped, _ = orc.token_terms(lp_minus_old, 0.0, A, 0.5, edge_lo if A < 0 else 0.2,
                                                edge_hi if A > 0 else 0.2, 1.0)
        assert unclipped and g == -0.5 * A * rho


def test_clip_fraction_counted_by_hand():
    """clip_frac = clipped tokens / tokens with a non-zero advantage (and weight), counted by hand:
    8 token rows; rollout 0 (A = +1) has ratios 1.0, 1.5 (clipped: above 1 + eps), 0.5 (not clipped:
    below the range but A > 0 keeps the unclipped branch); rollout 1 (A = -2) has ratios 0.5
    (clipped: below 1 - eps), 1.5 (not clipped for A < 0); rollout 2 has A = 0 (two tokens, one with
    a wild ratio) and one padding row: neither counts in the denominator.  2 of 5."""
    V = 6
    rng = np.random.default_rng(3)
    z = rng.normal(size=(8, V))
    y = np.array([0, 1, 2, 3, 4, 5, 0, 1], np.int32)
    tr = np.array([0, 0, 0, 1, 1, 2, 2, -1], np.int32)
    ratios = np.array([1.0, 1.5, 0.5, 0.5, 1.5, 9.0, 1.0, 9.0])
    lp = np.array([orc.logprob_row(z[t], y[t])[0] for t in range(8)])
    old = lp - np.log(ratios)
    adv, w = np.array([1.0, -2.0, 0.0]), np.array([0.5, 0.25, 0.125])
    out = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, 0.2, 0.2, z64=z)
    assert out["clip_frac"] == 2 / 5
    assert [bool(x) for x in out["g"] != 0] == [True, False, True, False, True, False, False, False]
    # loss by hand: -sum w min(rho A, clip(rho) A)
    want = -(0.5 * (1.0 + 1.2 + 0.5) + 0.25 * (-2.0) * (0.8 + 1.5))
    assert abs(out["loss"] - want) < 1e-12
    # a rollout with weight 0 leaves the count as well: 1 of 2
    out = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, np.array([0.0, 0.25, 0.125]), 0.2, 0.2, z64=z)
    assert out["clip_frac"] == 1 / 2
    # asymmetric range: eps_hi = 0.6 un-clips the 1.5 of rollout 0 -> 1 of 5
    out = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, 0.2, 0.6, z64=z)
    assert out["clip_frac"] == 1 / 5


def test_on_policy_loss_is_minus_mean_advantage():
    """With rho = 1 everywhere Eq. 2 gives J = mean over queries of the group mean of the
    advantages; arbitrary advantages are supplied, weights come from the curation step."""
    wl = ai.make_config("cfg3", Q=12, T=3000, V=40, len_lo=5, len_hi=60)
    for kw in (dict(), dict(reject_enable=1), dict(reject_enable=1, posterior_mode=1)):
        ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams(**kw))
        rng = np.random.default_rng(9)
        adv = rng.normal(size=wl.R) * ga["keep_mask"]
        # lay out every kept rollout in full so that the sequence mean is complete
        tr = np.concatenate([np.full(wl.lengths[i], i, np.int32) for i in range(wl.R)])
        T = len(tr)
        z = rng.normal(0, 3, size=(T, wl.V))
        y = rng.integers(0, wl.V, size=T).astype(np.int32)
        lp = np.array([orc.logprob_row(z[t], y[t])[0] for t in range(T)])
        out = orc.grpo_loss_bwd(None, "f64", wl.V, y, lp, tr, adv, ga["weight"], 0.2, 0.2,
                                want_dlogits=False, z64=z)
        off = wl.group_offsets
        want = 0.0
        for q in range(wl.Q):
            k = ga["keep_mask"][off[q]:off[q + 1]] == 1
            if k.any():
                want += adv[off[q]:off[q + 1]][k].mean()
        assert abs(out["loss"] + want / wl.Q) < 1e-12
        assert out["clip_frac"] == 0.0


def test_zero_variance_groups_cost_nothing():
    wl = ai.make_config("cfg1", V=32, L=4)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
    assert ga["zero_var"].tolist() == [1, 0, 1, 0]
    logits = wl.logits_rows(0, wl.T)
    lp, _, _ = orc.logprob_fwd(logits, "f32", wl.V, wl.targets)
    old = ai.draw_old_logprob(lp, wl.seed)
    out = orc.grpo_loss_bwd(logits, "f32", wl.V, wl.targets, old, wl.token_rollout, ga["adv"],
                            ga["weight"], 0.2, 0.2)
    dead = np.isin(wl.token_rollout, np.nonzero(ga["adv"] == 0)[0])
    assert dead.sum() == 2 * 8 * 4
    assert not out["dlogits"][dead].any() and not out["loss_terms"][dead].any()
    assert np.signbit(out["dlogits"][dead]).sum() == 0          # +0, not -0
    assert out["dlogits"][~dead].any()


def test_row_shift_and_vocabulary_relabelling_leave_the_step_unchanged():
    """A softmax policy (App. C) does not see a constant added to a row of logits, and renaming the
    vocabulary entries only renames the gradient's columns: log-prob, entropy, loss and clip fraction
    stay, lse moves by the constant, dlogits is permuted.  All optional terms on."""
    rng = np.random.default_rng(31)
    T, V, R = 40, 23, 6
    z = rng.normal(0, 3, size=(T, V))
    y = rng.integers(0, V, size=T).astype(np.int32)
    tr = rng.integers(-1, R, size=T).astype(np.int32)
    adv = rng.normal(size=R)
    adv[2] = 0.0
    w = rng.random(R) * 0.01
    base = [orc.logprob_row(z[t], y[t]) for t in range(T)]
    old = np.array([b[0] for b in base]) + rng.normal(0, 0.3, size=T)
    ref_lp = old + rng.normal(0, 0.2, size=T)
    kw = dict(grad_scale=3.0, entropy_coef=0.02, kl_coef=0.04, ref_logprob=ref_lp)
    out = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, 0.2, 0.2, z64=z, **kw)
    assert 0.0 < out["clip_frac"] < 1.0 and out["dlogits"].any()

    shift = rng.normal(0, 50, size=(T, 1))
    for t in range(T):
        lp, ent, lse = orc.logprob_row(z[t] + shift[t], y[t])
        assert abs(lp - base[t][0]) < 1e-12 and abs(ent - base[t][1]) < 1e-12
        assert abs(lse - base[t][2] - shift[t, 0]) < 1e-12
    shifted = orc.grpo_loss_bwd(None, "f64", V, y, old, tr, adv, w, 0.2, 0.2, z64=z + shift, **kw)
    assert abs(shifted["loss"] - out["loss"]) < 1e-14 and shifted["clip_frac"] == out["clip_frac"]
    assert np.abs(shifted["dlogits"] - out["dlogits"]).max() < 1e-13

    perm = rng.permutation(V)                   # new column j holds old column perm[j]
    inv = np.argsort(perm)
    renamed = orc.grpo_loss_bwd(None, "f64", V, inv[y].astype(np.int32), old, tr, adv, w, 0.2, 0.2,
                                z64=z[:, perm], **kw)
    assert abs(renamed["loss"] - out["loss"]) < 1e-14 and renamed["clip_frac"] == out["clip_frac"]
    assert np.abs(renamed["dlogits"] - out["dlogits"][:, perm]).max() < 1e-15
    # and the gradient rows of a softmax sum to zero over the vocabulary, with or without the extra terms
    assert np.abs(out["dlogits"].sum(axis=1)).max() < 1e-15


# ------------------------------------------------------------------ fused LM head

def test_fused_matches_autograd_through_the_matmul():
    wl = ai.make_config("cfg4", T=24, H=16, V=40, Q=2, len_lo=2, len_hi=6)
    h, W = wl.hidden_rows(0, wl.T), wl.weight_rows(0, wl.V)
    W = ai.f32_to_bf16_bits(orc.widen(W, "bf16").astype(np.float32) * 20)    # make logits O(1)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
    fwd = orc.lmhead_fused(h, W, wl.targets)
    old = ai.draw_old_logprob(fwd["logprob"], wl.seed, sigma=0.3)
    out = orc.lmhead_fused(h, W, wl.targets, old, wl.token_rollout, ga["adv"], ga["weight"], 0.2, 0.2, 1.0)

    ht = torch.tensor(orc.widen(h, "bf16"), requires_grad=True)
    Wt = torch.tensor(orc.widen(W, "bf16"), requires_grad=True)
    z = ht @ Wt.T
    lsm = torch.log_softmax(z, 1)
    lp = lsm.gather(1, torch.tensor(wl.targets, dtype=torch.int64)[:, None])[:, 0]
    assert np.allclose(fwd["logprob"], lp.detach().numpy(), atol=1e-13)
    assert np.allclose(fwd["entropy"], -(lsm.exp() * lsm).sum(1).detach().numpy(), atol=1e-12)
    tr = torch.tensor(np.maximum(wl.token_rollout, 0), dtype=torch.int64)
    valid = torch.tensor(wl.token_rollout >= 0)
    A, Wgt = torch.tensor(ga["adv"])[tr], torch.tensor(ga["weight"])[tr] * valid
    rho = torch.exp(lp - torch.tensor(old, dtype=torch.float64))
    loss = -(Wgt * torch.minimum(rho * A, torch.clamp(rho, 0.8, 1.2) * A)).sum()
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-13
    assert np.allclose(out["dhidden"], ht.grad.numpy(), rtol=1e-10, atol=1e-16)
    assert np.allclose(out["dweight"], Wt.grad.numpy(), rtol=1e-10, atol=1e-16)
    assert np.abs(out["dweight"].sum(axis=0)).max() < 1e-15      # dz rows sum to zero over the vocabulary
    dead = out["g"] == 0
    assert dead.any() and not out["dhidden"][dead].any()
