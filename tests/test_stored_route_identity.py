"""The algebra behind the fused backward pass that does not form the logits a second time, checked in float64
against the checker's own gradient rows (no GPU): with P_v = exp(z_v - z_y), scale = -g exp(logprob) and the
sampled token's entry replaced by -(exp(-logprob) - 1), the row scale * P is the checker's
dz = g (onehot - softmax(z)); and the two contractions follow with the scale moved out:
dhidden = scale * (P W),  dweight = P^T (scale * h)."""
import numpy as np

import aero_inputs as ai
from oracle import aero_oracle as orc


def test_scaled_exponentials_reproduce_the_gradient_rows():
    wl = ai.make_config("cfg4", T=96, H=32, V=300, Q=6, len_lo=1, len_hi=16)
    wl.sigma_w = 3.0 / np.sqrt(32)             # logits spread over tens of nats
    h, W = wl.hidden_rows(0, wl.T), wl.weight_rows(0, wl.V)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, orc.AdvParams())
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    fwd = orc.lmhead_fused(h, W, wl.targets)
    old = ai.draw_old_logprob(fwd["logprob"], wl.seed, sigma=0.3)
    ref = orc.lmhead_fused(h, W, wl.targets, old, wl.token_rollout, a32, w32, np.float32(0.2), np.float32(0.2), 1.0)
    z = orc.lmhead_logits(h, W)
    hf, Wf = orc.widen(h, "bf16"), orc.widen(W, "bf16")
    T, V = z.shape
    y = wl.targets
    rows = np.flatnonzero(ref["g"] != 0)
    assert rows.size > 10
    P = np.exp(z - z[np.arange(T), y][:, None])
    lp = fwd["logprob"]
    P[np.arange(T), y] = -np.expm1(-lp)
    scale = -ref["g"] * np.exp(lp)
    dz = scale[:, None] * P
    want = orc.grpo_loss_bwd(None, "f64", V, y, old, wl.token_rollout, a32, w32, np.float32(0.2), np.float32(0.2), 1.0,
                             want_dlogits=True, z64=z)["dlogits"]
    assert np.allclose(dz[rows], want[rows], rtol=1e-9, atol=1e-300)
    assert not want[np.setdiff1d(np.arange(T), rows)].any()
    assert np.allclose((scale[:, None] * (P @ Wf))[rows], ref["dhidden"][rows], rtol=1e-8, atol=1e-18)
    assert np.allclose(P[rows].T @ (scale[rows, None] * hf[rows]), ref["dweight"], rtol=1e-7, atol=1e-16)
