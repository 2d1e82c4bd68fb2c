"""Full-size parity, in the launch configuration bench.py times.

cfg2 and cfg3 (logits path, V = 151936): the checker runs the forward definition on every row
that matters (threaded over rows), so log-probs, entropy, the loss and the clip fraction are
compared in full; dlogits are compared on sampled rows plus padded / zero-advantage rows.
cfg4 and cfg5 (fused LM head): the float64 product is formed in row chunks for every row that
carries signal, so the loss, the clip fraction and the forward statistics are compared in full,
dweight element-wise on more than 4096 sampled vocabulary rows and dhidden on sampled tokens.
Each batch is also run with supplied one-signed advantages, where the loss must meet the stated
1e-4 relative tolerance with no rounding floor.
"""
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import aero_inputs as ai
from oracle import aero_oracle as orc
from oracle.aero_oracle import AdvParams

pytestmark = pytest.mark.gpu
THREADS = 16


@pytest.fixture(scope="module")
def gh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_helpers
    return gpu_helpers


def oracle_fwd_rows(host_rows, dtype, V, targets):
    """Checker forward on the given rows, threads over rows (numpy releases the GIL)."""
    n = host_rows.shape[0]
    out = np.zeros((n, 3))

    def one(i):
        out[i] = orc.logprob_row(orc.widen(host_rows[i, :V], dtype), int(targets[i]))

    with ThreadPoolExecutor(THREADS) as ex:
        list(ex.map(one, range(n)))
    return out


def logits_full_size(gh, name, params):
    wl = ai.make_config(name)
    T, V, ld = wl.T, wl.V, wl.ld
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams(**params))
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    tr = wl.token_rollout
    valid = tr >= 0
    signal = valid & (a32[np.maximum(tr, 0)] != 0) & (w32[np.maximum(tr, 0)] != 0)
    rng = np.random.default_rng(1234)
    sig_rows = np.nonzero(signal)[0]
    dead_rows = np.nonzero(~signal)[0]
    sampled = np.sort(np.concatenate([rng.choice(sig_rows, size=min(48, len(sig_rows)), replace=False),
                                      rng.choice(dead_rows, size=min(16, len(dead_rows)), replace=False)
                                      if len(dead_rows) else np.zeros(0, np.int64)])).astype(np.int64)
    keep_host = {}
    logits = torch.empty((T, ld), dtype=torch.bfloat16, device=gh.DEV)
    ref = np.zeros((T, 3))
    chunk = 2048
    for r0 in range(0, T, chunk):
        r1 = min(T, r0 + chunk)
        h = wl.logits_rows(r0, r1, threads=THREADS)
        logits[r0:r1].copy_(torch.from_numpy(h.view(np.int16)).view(torch.bfloat16))
        rows = np.nonzero(valid[r0:r1])[0]
        ref[r0 + rows] = oracle_fwd_rows(h[rows], wl.dtype, V, wl.targets[r0 + rows])
        for t in sampled[(sampled >= r0) & (sampled < r1)]:
            keep_host[int(t)] = h[t - r0].copy()
    lp_ref, ent_ref, lse_ref = ref[:, 0], ref[:, 1], ref[:, 2]

    # forward, as bench.py calls it
    active = valid.astype(np.uint8)
    lp, ent, lse, err = gh.run_fwd(logits, T, V, ld, wl.targets, active)
    assert err == 0
    for got, want in ((lp, lp_ref), (ent, ent_ref), (lse, lse_ref)):
        g = got.cpu().numpy().astype(np.float64)
        assert np.abs(g - want).max() <= 2e-3
        assert not g[~valid].any()

    # loss + dlogits with the library's own lse, as bench.py calls it
    old = ai.draw_old_logprob(lp_ref, wl.seed, sigma=0.05)
    eps = np.float32(wl.eps)
    loss_ref, n_sig, n_clip = 0.0, 0, 0
    terms = []
    g_ref = np.zeros(T)
    for t in sig_rows:
        term, g_ref[t], unclipped, _ = orc.token_terms(lp_ref[t], float(old[t]), float(a32[tr[t]]), float(w32[tr[t]]),
                                                       float(eps), float(eps), 1.0)
        loss_ref += term
        terms.append(term)
        n_sig += 1
        n_clip += 0 if unclipped else 1
    out = gh.run_loss_bwd(logits, T, V, ld, wl.targets, lse, old, tr, ga["adv"], ga["weight"], eps=float(eps))
    assert out["err"] == 0
    gh.assert_loss(out["loss"].item(), loss_ref, terms)
    assert abs(out["clip_frac"].item() - (n_clip / n_sig if n_sig else 0.0)) < 1e-6
    lp_out = out["logprob"].cpu().numpy().astype(np.float64)
    assert np.abs(lp_out[signal] - lp_ref[signal]).max() <= 2e-3 and not lp_out[~signal].any()

    sel = sampled
    host_sel = np.stack([keep_host[int(t)] for t in sel])
    sub = orc.grpo_loss_bwd(host_sel, wl.dtype, V, wl.targets[sel], old[sel], tr[sel], a32, w32, eps, eps, 1.0)
    dz = out["dlogits"][torch.from_numpy(sel).to(gh.DEV)].float().cpu().numpy().astype(np.float64)[:, :V]
    want = sub["dlogits"]
    assert np.abs(dz - want).max() <= 1e-2
    assert (np.abs(dz - want) <= 1e-2 * np.abs(sub["g"])[:, None] + np.abs(want) * 2.0 ** -8 + 1e-30).all()
    dead_sel = sub["g"] == 0
    assert not dz[dead_sel].any()
    # every row without signal is exactly +0 in the whole tensor
    nz_rows = (out["dlogits"].view(torch.int16) != 0).any(dim=1).cpu().numpy()
    assert not nz_rows[~signal].any() and nz_rows[g_ref != 0].all()

    # the same step as the one-call route the bench times: statistics, loss and gradient in one
    # pass, log-prob / entropy / lse written for every valid row
    del out
    torch.cuda.empty_cache()
    one = gh.run_loss_bwd(logits, T, V, ld, wl.targets, None, old, tr, ga["adv"], ga["weight"], eps=float(eps),
                          stats=True)
    assert one["err"] == 0
    gh.assert_loss(one["loss"].item(), loss_ref, terms)
    assert abs(one["clip_frac"].item() - (n_clip / n_sig if n_sig else 0.0)) < 1e-6
    valid = active.astype(bool)
    for key, want_all in (("logprob", lp_ref), ("entropy", ent_ref), ("lse", lse_ref)):
        got = one[key].cpu().numpy().astype(np.float64)
        assert np.abs(got[valid] - want_all[valid]).max() <= 2e-3 and not got[~valid].any(), key
    dz1 = one["dlogits"][torch.from_numpy(sel).to(gh.DEV)].float().cpu().numpy().astype(np.float64)[:, :V]
    assert (np.abs(dz1 - want) <= 1e-2 * np.abs(sub["g"])[:, None] + np.abs(want) * 2.0 ** -8 + 1e-30).all()
    nz_rows = (one["dlogits"].view(torch.int16) != 0).any(dim=1).cpu().numpy()
    assert not nz_rows[~signal].any() and nz_rows[g_ref != 0].all()

    # padding rows marked "leave the gradient row alone": those rows keep the buffer's contents, every other
    # row, the loss and the statistics come out bit for bit as with plain padding (both routes)
    pads = np.nonzero(tr < 0)[0]
    if pads.size:
        tr_u = np.where(tr < 0, gh.binding.AERO_ROW_UNTOUCHED, tr).astype(np.int32)
        pads_d, rest_d = torch.from_numpy(pads).to(gh.DEV), torch.from_numpy(np.nonzero(tr >= 0)[0]).to(gh.DEV)
        for lse_arg in (None, lse):
            u = gh.run_loss_bwd(logits, T, V, ld, wl.targets, lse_arg, old, tr_u, ga["adv"], ga["weight"],
                                eps=float(eps), stats=lse_arg is None)
            assert u["err"] == 0
            if lse_arg is None:
                assert u["loss"].item() == one["loss"].item()
            else:       # the forward call's lse differs from the single-pass one by fp32 rounding
                gh.assert_loss(u["loss"].item(), loss_ref, terms)
            assert gh.all_seven(u["dlogits"][pads_d])
            assert torch.equal(u["dlogits"][rest_d].view(torch.int16), one["dlogits"][rest_d].view(torch.int16)) \
                if lse_arg is None else \
                bool(((u["dlogits"][rest_d].float() - one["dlogits"][rest_d].float()).abs()
                      <= 2.0 ** -7 * one["dlogits"][rest_d].float().abs() + 1e-12).all())
            if lse_arg is None:
                for key in ("logprob", "entropy", "lse"):
                    assert torch.equal(u[key], one[key]), key
            del u
    del one
    torch.cuda.empty_cache()

    # supplied advantages of one sign on every rollout: nothing cancels in the loss, so the stated
    # tolerance (1e-4 relative) holds with no rounding floor; loss-only calls on both routes
    a_pos = (np.abs(a32) + np.float32(0.25)).astype(np.float32)
    terms = np.zeros(T)
    n_clip = 0
    all_sig = np.nonzero(valid & (w32[np.maximum(tr, 0)] != 0))[0]
    for t in all_sig:
        terms[t], _, unclipped, _ = orc.token_terms(lp_ref[t], float(old[t]), float(a_pos[tr[t]]), float(w32[tr[t]]),
                                                    float(eps), float(eps), 1.0)
        n_clip += 0 if unclipped else 1
    for lse_arg in (lse, None):
        o = gh.run_loss_bwd(logits, T, V, ld, wl.targets, lse_arg, old, tr, a_pos, ga["weight"], eps=float(eps),
                            want_dlogits=False)
        gh.assert_loss(o["loss"].item(), float(terms.sum()), terms, strict=True)
        assert abs(o["clip_frac"].item() - n_clip / len(all_sig)) < 1e-6
    return wl


def test_cfg2_full_size(gh):
    wl = logits_full_size(gh, "cfg2", dict())
    assert wl.T == 16384 and wl.V == 151936


def test_cfg3_full_size(gh):
    wl = logits_full_size(gh, "cfg3", dict())
    assert wl.T == 32768 and wl.V == 151936


def fused_full_size(gh, name, n_dh):
    """Every row that carries signal goes through the float64 product (row chunks), so the loss, the
    clip fraction and the forward statistics are compared in full; dweight is compared element-wise
    on more than 4096 sampled vocabulary rows (sampled-token rows, chunk edges and the ragged end
    of the vocabulary among them), dhidden on sampled tokens."""
    from test_gpu_fused import run_fused, rowwise_close
    from fused_reference import fused_reference, sample_vocab_rows
    wl = ai.make_config(name)
    T, H, V = wl.T, wl.H, wl.V
    h = wl.hidden_rows(0, T, threads=THREADS)
    W = wl.weight_rows(0, V, threads=THREADS)
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams())
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    tr = wl.token_rollout
    signal = (tr >= 0) & (a32[np.maximum(tr, 0)] != 0) & (w32[np.maximum(tr, 0)] != 0)
    rng = np.random.default_rng(4321)
    sig_rows, dead_rows = np.nonzero(signal)[0], np.nonzero(~signal)[0]
    dh_rows = np.sort(np.concatenate([rng.choice(sig_rows, size=n_dh, replace=False),
                                      rng.choice(dead_rows, size=8, replace=False)]))
    v_sel = sample_vocab_rows(wl, sig_rows, rng)
    assert len(v_sel) >= 4096
    print("%s: float64 reference over %d rows, %d vocabulary rows" % (name, len(sig_rows), len(v_sel)), flush=True)
    ref = fused_reference(wl, h, W, a32, w32, v_sel, dh_rows, sigma_old=0.05, threads=THREADS)
    print("%s: reference done, clip_frac %.4f" % (name, ref["clip_frac"]), flush=True)

    out = run_fused(gh, wl, h, W, wl.targets, bwd=dict(old=ref["old"], adv=a32, weight=w32),
                    dweight_dtype=torch.bfloat16)
    assert out["err"] == 0
    rows = ref["rows"]
    for k, want in (("logprob", ref["lp"]), ("entropy", ref["ent"]), ("lse", ref["lse"])):
        got = out[k].cpu().numpy().astype(np.float64)[rows]
        assert np.abs(got - want).max() <= 2e-3, k
    ratio = gh.assert_loss(out["loss"].item(), ref["loss"], ref["loss_terms"])
    assert abs(out["clip_frac"].item() - ref["clip_frac"]) < 1e-6
    # dweight, sampled vocabulary rows: |diff| <= 1e-2 of the row's largest reference entry
    dw = out["dweight"][torch.from_numpy(v_sel).to(gh.DEV)].float().cpu().numpy().astype(np.float64)
    assert np.abs(ref["dweight_sel"]).max(axis=1).min() > 0
    assert rowwise_close(dw, ref["dweight_sel"])
    # dhidden, sampled tokens
    dh = out["dhidden"][torch.from_numpy(dh_rows).to(gh.DEV)].float().cpu().numpy().astype(np.float64)
    for i, t in enumerate(dh_rows):
        want = ref["dhidden"][int(t)]
        if ref["g"][t] == 0:
            assert not dh[i].any() and not want.any()
        else:
            assert np.abs(dh[i] - want).max() <= 1e-2 * np.abs(want).max() + 1e-30
    # every token without gradient has an exactly +0 dhidden row
    nz = (out["dhidden"].view(torch.int16) != 0).any(dim=1).cpu().numpy()
    assert not nz[ref["g"] == 0].any() and nz[ref["g"] != 0].all()
    assert torch.isfinite(out["dweight"].float()).all()
    del out
    torch.cuda.empty_cache()

    # the same batch with supplied advantages of one sign: nothing cancels in the loss, so the
    # stated tolerance (1e-4 relative) holds with no rounding floor
    a_pos = np.where(a32 != 0, np.abs(a32), 0).astype(np.float32)
    pos = {int(t): i for i, t in enumerate(rows)}
    terms = np.zeros(T)
    for t in sig_rows:
        terms[t] = orc.token_terms(ref["lp"][pos[int(t)]], float(ref["old"][t]), float(a_pos[tr[t]]), float(w32[tr[t]]),
                                   float(np.float32(0.2)), float(np.float32(0.2)), 1.0)[0]
    out = run_fused(gh, wl, h, W, wl.targets, bwd=dict(old=ref["old"], adv=a_pos, weight=w32),
                    dweight_dtype=torch.bfloat16)
    gh.assert_loss(out["loss"].item(), float(terms.sum()), terms, strict=True)
    return ratio


def test_cfg4_full_size(gh):
    fused_full_size(gh, "cfg4", 40)


def test_cfg5_full_size(gh):
    fused_full_size(gh, "cfg5", 24)
