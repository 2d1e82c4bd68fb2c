"""Float64 reference of the fused LM-head step at sizes where the [T, V] logits cannot be held
at once: the checker's definitions (oracle.aero_oracle) applied to row chunks of the float64
product.  Test infrastructure: imports the checker, never the GPU library.

What it returns for a workload (hidden h, weight W as bf16 bit patterns):
  * lp / ent / lse of every row in `rows` (the rows that carry signal plus any extra rows),
  * the behaviour log-probs it drew from those (seeded noise; constant stand-in elsewhere),
  * loss, clip fraction, per-token loss terms and g_t over all tokens (Eq. 2),
  * dweight[v_sel, :] = sum_t dz[t, v_sel] h[t] for the sampled vocabulary rows v_sel, with
    dz[t, j] = g_t (1[j = y_t] - exp(z[t, j] - lse_t)) unrounded (App. A.1),
  * dhidden[t, :] = dz[t, :] W for the rows in `dh_rows`.
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import aero_inputs as ai
from oracle import aero_oracle as orc


def fused_reference(wl, h_bits, W_bits, adv32, weight32, v_sel, dh_rows, extra_rows=(), sigma_old=0.05,
                    eps=0.2, grad_scale=1.0, chunk=512, threads=16):
    T, V = wl.T, wl.V
    tr, y = wl.token_rollout, wl.targets
    ri = np.maximum(tr, 0)
    signal = (tr >= 0) & (y >= 0) & (adv32[ri] != 0) & (weight32[ri] != 0)
    rows = np.unique(np.concatenate([np.nonzero(signal)[0], np.asarray(extra_rows, np.int64),
                                     np.asarray(dh_rows, np.int64)])).astype(np.int64)
    v_sel = np.asarray(v_sel, np.int64)
    W64 = orc.widen(W_bits, "bf16")            # [V, H]
    h64 = orc.widen(h_bits[rows], "bf16")      # [n, H]
    n = len(rows)
    stats = np.zeros((n, 3))                   # lp, ent, lse per row of `rows`
    z_sel = np.zeros((n, len(v_sel)))          # logits at the sampled vocabulary columns
    keep = {int(t): None for t in dh_rows}     # full logits rows of the dhidden sample

    with ThreadPoolExecutor(threads) as ex:
        for c0 in range(0, n, chunk):
            c1 = min(n, c0 + chunk)
            z = h64[c0:c1] @ W64.T             # the float64 product, rows c0..c1

            def one(i):
                stats[c0 + i] = orc.logprob_row(z[i], int(y[rows[c0 + i]]))

            list(ex.map(one, range(c1 - c0)))
            z_sel[c0:c1] = z[:, v_sel]
            for i in range(c1 - c0):
                t = int(rows[c0 + i])
                if t in keep:
                    keep[t] = z[i].copy()

    lp_all = np.full(T, -math.log(V))          # stand-in where no token term is formed
    lp_all[rows] = stats[:, 0]
    old = ai.draw_old_logprob(lp_all, wl.seed, sigma=sigma_old, eps_lo=eps, eps_hi=eps)

    e32 = float(np.float32(eps))
    g = np.zeros(T)
    terms = np.zeros(T)
    n_sig = n_clip = 0
    pos_of = {int(t): i for i, t in enumerate(rows)}
    for t in np.nonzero(signal)[0]:
        i = pos_of[int(t)]
        terms[t], g[t], unclipped, _ = orc.token_terms(stats[i, 0], float(old[t]), float(adv32[tr[t]]),
                                                       float(weight32[tr[t]]), e32, e32, grad_scale)
        n_sig += 1
        n_clip += 0 if unclipped else 1
    loss = float(terms.sum())

    # dweight rows: dz[:, v_sel]^T h
    g_rows = g[rows]
    dz_sel = -g_rows[:, None] * np.exp(z_sel - stats[:, 2][:, None])
    col_of = {int(v): k for k, v in enumerate(v_sel)}
    for i, t in enumerate(rows):
        k = col_of.get(int(y[t]))
        if k is not None:
            dz_sel[i, k] += g_rows[i]
    dW_sel = dz_sel.T @ h64

    dh = {}
    for t in dh_rows:
        t = int(t)
        i = pos_of[t]
        row = -g[t] * np.exp(keep[t] - stats[i, 2])
        row[int(y[t])] += g[t]
        dh[t] = row @ W64
    return dict(rows=rows, signal=signal, lp=stats[:, 0], ent=stats[:, 1], lse=stats[:, 2], old=old, g=g,
                loss_terms=terms, loss=loss, clip_frac=(n_clip / n_sig if n_sig else 0.0), dweight_sel=dW_sel,
                dhidden=dh)


def sample_vocab_rows(wl, grad_rows, rng, n_random=4096, n_targets=64, tail=300):
    """Vocabulary rows for the dweight comparison: random ones, the sampled-token rows of some
    tokens with gradient (where the onehot term lands), the rows next to every multiple of 32768
    (the backward pass walks the vocabulary in chunks of such multiples) and the last `tail` rows
    (short last chunk, ragged last tile)."""
    V = wl.V
    parts = [rng.choice(V, size=min(n_random, V), replace=False)]
    if len(grad_rows):
        parts.append(wl.targets[rng.choice(grad_rows, size=min(n_targets, len(grad_rows)), replace=False)])
    edges = np.arange(0, V, 32768)
    parts.append(np.concatenate([edges, edges[1:] - 1, edges + 1]))
    parts.append(np.arange(max(0, V - tail), V))
    v = np.unique(np.concatenate(parts).astype(np.int64))
    return v[(v >= 0) & (v < V)]
