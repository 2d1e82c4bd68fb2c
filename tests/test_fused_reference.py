"""The chunked float64 reference that the full-size fused parity tests use must be the checker's
plain definition (whole [T, V] product at once) evaluated piecewise: compared here on a shape
small enough for both, with chunks that do not divide the row count."""
import numpy as np

import aero_inputs as ai
from oracle import aero_oracle as orc
from fused_reference import fused_reference, sample_vocab_rows


def test_chunked_reference_equals_the_plain_definition():
    wl = ai.make_config("cfg5", T=700, H=64, V=3000, Q=48, len_lo=1, len_hi=40)
    wl.sigma_w = 0.25
    h, W = wl.hidden_rows(0, wl.T), wl.weight_rows(0, wl.V)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, orc.AdvParams())
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    rng = np.random.default_rng(9)
    tr = wl.token_rollout
    sig = np.nonzero((tr >= 0) & (a32[np.maximum(tr, 0)] != 0))[0]
    dead = np.nonzero(~((tr >= 0) & (a32[np.maximum(tr, 0)] != 0)))[0]
    assert len(sig) > 100 and len(dead) > 10
    v_sel = sample_vocab_rows(wl, sig, rng, n_random=200, n_targets=16, tail=40)
    dh_rows = np.sort(np.concatenate([rng.choice(sig, 12, replace=False), dead[:3]]))
    ref = fused_reference(wl, h, W, a32, w32, v_sel, dh_rows, extra_rows=dead[3:6], sigma_old=0.3, chunk=97,
                          threads=4)
    assert 0.02 < ref["clip_frac"] < 0.98
    plain = orc.lmhead_fused(h, W, wl.targets, ref["old"], tr, a32, w32, np.float32(0.2), np.float32(0.2), 1.0)
    rows = ref["rows"]
    for k in ("lp", "ent", "lse"):
        assert np.allclose(ref[k], plain[{"lp": "logprob", "ent": "entropy", "lse": "lse"}[k]][rows], rtol=0, atol=1e-12)
    assert np.allclose(ref["g"], plain["g"], rtol=1e-12, atol=0)
    assert np.allclose(ref["loss_terms"], plain["loss_terms"], rtol=1e-12, atol=0)
    assert abs(ref["loss"] - plain["loss"]) <= 1e-12 * np.abs(plain["loss_terms"]).sum()
    assert ref["clip_frac"] == plain["clip_frac"]
    scale = np.abs(plain["dweight"]).max()
    assert np.abs(ref["dweight_sel"] - plain["dweight"][v_sel]).max() <= 1e-12 * scale
    for t in dh_rows:
        assert np.abs(ref["dhidden"][int(t)] - plain["dhidden"][t]).max() <= 1e-12 * np.abs(plain["dhidden"]).max()
    assert not any(ref["dhidden"][int(t)].any() for t in dead[:3])
    # the vocabulary sample contains what it is meant to cover
    assert wl.V - 1 in v_sel and 0 in v_sel and np.isin(wl.targets[sig], v_sel).sum() >= 16
