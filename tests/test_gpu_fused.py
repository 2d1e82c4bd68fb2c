"""GPU parity for the LM-head-fused path: statistics without materialised logits, loss, and
the gradients w.r.t. hidden states and LM-head weight, against the float64 checker (which
forms the logits as a float64 product and then applies the logits-path definitions).

Tolerances: log-prob / entropy / lse 2e-3 absolute; loss 1e-4 relative (plus an fp32 rounding floor only where the terms cancel, see gpu_helpers.loss_bound); gradients are checked
scale-free, per row, against 1e-2 of the largest reference entry of that row (the operands of
the two gradient contractions are rounded to bf16, dhidden is stored in bf16); a dweight
requested in bf16 is allowed the rounding of its own stored entries, 2^-8 relative, on top."""
import numpy as np
import pytest
import torch

import aero_inputs as ai
from oracle import aero_oracle as orc
from oracle.aero_oracle import AdvParams

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_helpers
    return gpu_helpers


def run_fused(gh, wl, h_bits, w_bits, targets, bwd=None, dweight_dtype=torch.float32, dw_into=None):
    """dw_into: a dweight buffer to accumulate into (AERO_DW_ACCUMULATE) instead of a fresh one."""
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding
    dev = gh.DEV
    T, H, V = wl.T, wl.H, wl.V
    hd = torch.from_numpy(h_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    wd = torch.from_numpy(w_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    lp, ent, lse = (torch.full((T,), 7.0, device=dev) for _ in range(3))
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=T, V=V, H=H, R=wl.R), dtype=torch.uint8,
                     device=dev)
    out = dict(logprob=lp, entropy=ent, lse=lse)
    if bwd is None:
        aero.aero_lmhead_logprob_fused(hd, wd, T, H, V, gh.dev(targets), lp, ent, lse, workspace=ws, err_flag=err)
    else:
        loss, clip = torch.full((1,), 7.0, device=dev), torch.full((1,), 7.0, device=dev)
        dh = torch.full((T, H), 7.0, dtype=torch.bfloat16, device=dev)
        dw = torch.full((V, H), 7.0, dtype=dweight_dtype, device=dev) if dw_into is None else dw_into
        aero.aero_lmhead_logprob_fused(
            hd, wd, T, H, V, gh.dev(targets), lp, ent, lse, gh.dev(bwd["old"].astype(np.float32)),
            gh.dev(wl.token_rollout), gh.dev(bwd["adv"].astype(np.float32)), gh.dev(bwd["weight"].astype(np.float32)),
            wl.R, 0.2, 0.2, bwd.get("grad_scale", 1.0), loss, clip, dh, dw, ws, err,
            entropy_coef=bwd.get("entropy_coef", 0.0), kl_coef=bwd.get("kl_coef", 0.0),
            ref_logprob=gh.dev(bwd["ref_lp"].astype(np.float32)) if bwd.get("ref_lp") is not None else None,
            dweight_accumulate=dw_into is not None)
        out.update(loss=loss, clip_frac=clip, dhidden=dh, dweight=dw)
    torch.cuda.synchronize()
    out["err"] = int(err.item())
    return out


def make(T, H, V, Q=6, sigma_w=None, name="cfg4", seed=None, len_hi=None):
    wl = ai.make_config(name, T=T, H=H, V=V, Q=Q, len_lo=1, len_hi=len_hi or max(2, T // 6), seed=seed)
    if sigma_w is not None:
        wl.sigma_w = sigma_w
    return wl, wl.hidden_rows(0, T), wl.weight_rows(0, V)


def rowwise_close(got, want, frac=1e-2, stored_rounding=0.0):
    """stored_rounding: relative rounding of the stored entry itself, allowed on top (2^-8 for a dweight the
    caller asks for in bf16; over a vocabulary of 2^18 rows the tail of the operand-rounding noise comes within
    a tenth of the row bound, and the output's own rounding is a separate, known quantity)."""
    scale = np.abs(want).max(axis=1, keepdims=True)
    return (np.abs(got - want) <= frac * scale + stored_rounding * np.abs(want) + 1e-30).all()


# (300, 2112, 1000): 33 K slices, the contraction loop's L2 warm-up (from 32 slices on) is active
FWD_SHAPES = [(256, 64, 256), (300, 64, 1000), (17, 72, 77), (512, 1536, 3000), (700, 512, 5001 - 1),
              (1, 8, 1), (1100, 256, 4096), (300, 2112, 1000)]


@pytest.mark.parametrize("T,H,V", FWD_SHAPES)
def test_fused_forward(gh, T, H, V):
    wl, h, W = make(T, H, V, sigma_w=2.0 / np.sqrt(H))
    tg = wl.targets.copy()
    if T > 4:
        tg[3] = -1
    ref = orc.lmhead_fused(h, W, tg)
    out = run_fused(gh, wl, h, W, tg)
    assert out["err"] == 0
    for k in ("logprob", "entropy", "lse"):
        got = out[k].cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        assert np.abs(got - ref[k]).max() <= 2e-3, k
        assert not got[tg < 0].any()


def check_bwd(gh, wl, h, W, params, sigma_old=0.3, dweight_dtype=torch.float32, grad_scale=1.0, entropy_coef=0.0,
              kl_coef=0.0, adv_map=None, strict_loss=False):
    """adv_map / strict_loss: supplied advantages and the pure 1e-4 relative loss bound, as in the
    logits-path tests."""
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams(**params))
    if adv_map is not None:
        ga["adv"] = adv_map(ga["adv"].astype(np.float32)).astype(np.float64)
    fwd = orc.lmhead_fused(h, W, wl.targets)
    old = ai.draw_old_logprob(fwd["logprob"], wl.seed, sigma=sigma_old)
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    ref_lp = (old + np.random.default_rng(wl.seed + 77).normal(0, 0.2, size=old.shape)).astype(np.float32) \
        if kl_coef != 0.0 else None
    ref = orc.lmhead_fused(h, W, wl.targets, old, wl.token_rollout, a32, w32, np.float32(0.2), np.float32(0.2),
                           grad_scale, entropy_coef=entropy_coef, kl_coef=kl_coef, ref_logprob=ref_lp)
    out = run_fused(gh, wl, h, W, wl.targets,
                    bwd=dict(old=old, adv=a32, weight=w32, grad_scale=grad_scale, entropy_coef=entropy_coef,
                             kl_coef=kl_coef, ref_lp=ref_lp),
                    dweight_dtype=dweight_dtype)
    assert out["err"] == 0
    gh.assert_loss(out["loss"].item(), ref["loss"], ref["loss_terms"], strict=strict_loss)
    assert abs(out["clip_frac"].item() - ref["clip_frac"]) < 1e-6
    dh = out["dhidden"].float().cpu().numpy().astype(np.float64)
    dw = out["dweight"].float().cpu().numpy().astype(np.float64)
    assert np.isfinite(dh).all() and np.isfinite(dw).all()
    assert rowwise_close(dh, ref["dhidden"])
    assert rowwise_close(dw, ref["dweight"], stored_rounding=2.0 ** -8 if dweight_dtype == torch.bfloat16 else 0.0)
    dead = (ref["g"] == 0) & (ref["e"] == 0)
    assert not out["dhidden"].view(torch.int16)[torch.from_numpy(dead).to(gh.DEV)].any()   # +0 rows
    return ref, out


# the last two reach 32 K slices in the recompute (H = 2112) and in the dweight contraction (> 2048 tokens
# with gradient), where the loop warms L2 ahead of its operand requests; then 1024 vocabulary tiles, and a hidden size of 8192
@pytest.mark.parametrize("T,H,V", [(256, 64, 256), (300, 64, 1000), (17, 72, 77), (700, 512, 5000),
                                   (512, 1536, 3000), (1100, 256, 4096), (300, 2112, 1000), (4500, 64, 600),
                                   (300, 64, 262144), (130, 8192, 700)])
def test_fused_backward(gh, T, H, V):
    wl, h, W = make(T, H, V, sigma_w=2.0 / np.sqrt(H))
    ref, _ = check_bwd(gh, wl, h, W, dict())
    assert (ref["g"] != 0).any()
    if T >= 4096:
        assert (ref["g"] != 0).sum() > 2048
    check_bwd(gh, wl, h, W, dict(reject_enable=1, posterior_mode=1), dweight_dtype=torch.bfloat16, grad_scale=8.0)


@pytest.mark.parametrize("seed", range(10))
def test_fused_random_shapes(gh, seed):
    """Seeded random token counts, hidden sizes (multiples of 8, with and without whole 64-wide K slices)
    and vocabulary sizes (ragged last tile), both workload kinds, random call variants."""
    rng = np.random.default_rng(3000 + seed)
    T = int(rng.choice([rng.integers(1, 40), rng.integers(40, 600), rng.integers(600, 1500)]))
    H = 8 * int(rng.choice([rng.integers(1, 9), rng.integers(9, 80)]))
    V = int(rng.choice([rng.integers(2, 300), rng.integers(300, 6000)]))
    name = ["cfg4", "cfg5"][seed % 2]
    wl, h, W = make(T, H, V, Q=int(rng.integers(2, 12)), sigma_w=2.0 / np.sqrt(H), name=name, seed=50 + seed,
                    len_hi=max(2, T // int(rng.integers(2, 9))))
    tg = wl.targets.copy()
    if T > 8:
        tg[rng.integers(0, T, size=3)] = -1          # rows without a target take no part
    ref = orc.lmhead_fused(h, W, tg)
    out = run_fused(gh, wl, h, W, tg)
    assert out["err"] == 0
    for k in ("logprob", "entropy", "lse"):
        got = out[k].cpu().numpy().astype(np.float64)
        assert np.abs(got - ref[k]).max() <= 2e-3 and not got[tg < 0].any(), k
    terms = rng.random() < 0.5
    check_bwd(gh, wl, h, W, dict(reject_enable=int(rng.integers(2)), posterior_mode=int(rng.integers(2))),
              sigma_old=float(rng.choice([0.05, 0.3])),
              dweight_dtype=[torch.float32, torch.bfloat16][int(rng.integers(2))],
              grad_scale=float(rng.choice([1.0, 8.0])), entropy_coef=0.01 if terms else 0.0,
              kl_coef=0.04 if terms and rng.random() < 0.5 else 0.0)


@pytest.mark.parametrize("z_std", [5.0, 25.0])
def test_fused_backward_wide_logits(gh, z_std):
    """Logits spread so widely that sampled tokens lie tens of nats (z_std = 5: up to 33) or more than the stored
    exponentials' safe range of 40 (z_std = 25: up to 165) below the row maximum.  The first stays on the
    route that reuses the forward pass's exponentials, the second makes the forward pass raise its flag and the
    backward pass recompute the logits; both must match the checker."""
    T, H, V = 520, 128, 3000
    wl, h, W = make(T, H, V, sigma_w=z_std / np.sqrt(H))
    z = orc.lmhead_logits(h, W)
    gap = z.max(axis=1) - z[np.arange(T), wl.targets]
    assert (gap.max() > 40.0) == (z_std > 20.0) and gap.max() > 30.0
    check_bwd(gh, wl, h, W, dict())
    check_bwd(gh, wl, h, W, dict(reject_enable=1, posterior_mode=1), dweight_dtype=torch.bfloat16, grad_scale=8.0,
              kl_coef=0.04)


def test_fused_backward_several_chunks_and_recipe_scale(gh):
    """Vocabulary wider than one backward chunk at this T (2 x 24576 > chunk), paper-scale weights."""
    wl, h, W = make(2816, 128, 40000, Q=8, len_hi=500)
    check_bwd(gh, wl, h, W, dict(), sigma_old=0.05)


def test_fused_entropy_bonus(gh):
    """Entropy bonus through the fused path: more rows carry gradient (advantage-0 rollouts with a
    weight), loss and both gradients follow the checker."""
    wl, h, W = make(520, 128, 1000, sigma_w=0.3)
    ref0, _ = check_bwd(gh, wl, h, W, dict())
    for coef in (1e-3, 0.05):
        ref, _ = check_bwd(gh, wl, h, W, dict(), entropy_coef=coef)
        assert (ref["e"] != 0).sum() > (ref0["g"] != 0).sum() and ref["loss"] < ref0["loss"]
    check_bwd(gh, wl, h, W, dict(reject_enable=1, posterior_mode=1), entropy_coef=0.01, dweight_dtype=torch.bfloat16,
              grad_scale=8.0)
    wl, h, W = make(2816, 128, 40000, Q=8, len_hi=500)     # several vocabulary chunks
    check_bwd(gh, wl, h, W, dict(), sigma_old=0.05, entropy_coef=1e-3)


def test_fused_kl_penalty(gh):
    wl, h, W = make(520, 128, 1000, sigma_w=0.3)
    ref0, _ = check_bwd(gh, wl, h, W, dict())
    ref, _ = check_bwd(gh, wl, h, W, dict(), kl_coef=0.04)
    assert ref["loss"] > ref0["loss"] and (ref["g"] != 0).sum() > (ref0["g"] != 0).sum()
    check_bwd(gh, wl, h, W, dict(reject_enable=1, posterior_mode=1), kl_coef=0.04, entropy_coef=1e-3,
              dweight_dtype=torch.bfloat16, grad_scale=8.0)


@pytest.mark.parametrize("T,H,V", [(700, 512, 5000), (300, 2112, 1000)])
def test_fused_loss_strict_tolerance(gh, T, H, V):
    """One-signed terms (supplied advantages of one sign; all-wrong groups in posterior mode): the
    loss meets the stated 1e-4 relative tolerance with no rounding floor."""
    wl, h, W = make(T, H, V, sigma_w=2.0 / np.sqrt(H))
    check_bwd(gh, wl, h, W, dict(), adv_map=lambda a: np.abs(a) + np.float32(0.25), strict_loss=True)
    check_bwd(gh, wl, h, W, dict(), sigma_old=0.05, adv_map=lambda a: -np.abs(a) - np.float32(0.25), strict_loss=True)
    wl.rewards[:] = 0.0
    ref, _ = check_bwd(gh, wl, h, W, dict(reject_enable=1, posterior_mode=1), strict_loss=True)
    assert (ref["g"] != 0).any() and ref["loss"] > 0


def test_fused_all_groups_zero_variance(gh):
    wl, h, W = make(300, 64, 1000, sigma_w=0.25)
    wl.rewards[:] = 1.0
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, None, AdvParams())
    assert not ga["adv"].any()
    old = np.full(wl.T, -5.0, np.float32)
    out = run_fused(gh, wl, h, W, wl.targets, bwd=dict(old=old, adv=ga["adv"], weight=ga["weight"]))
    assert out["loss"].item() == 0.0
    assert not out["dhidden"].view(torch.int16).any() and not out["dweight"].any()


def test_fused_rows_outside_every_rollout(gh):
    """Token rows with a target but no usable rollout (padding index, untouched mark, index past R): their
    statistics are still computed, they take no part in the gradient contractions, their dhidden rows are +0,
    and only the index past R raises the device error bit; the other rows match the checker."""
    from paper_2602_14338_amd import binding
    wl, h, W = make(520, 128, 1000, sigma_w=0.3)
    tr = wl.token_rollout.copy()
    tr[5], tr[6], tr[300] = -1, binding.AERO_ROW_UNTOUCHED, wl.R + 3
    tr_ref = tr.copy()
    tr_ref[[5, 6, 300]] = -1
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams())
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    fwd = orc.lmhead_fused(h, W, wl.targets)
    old = ai.draw_old_logprob(fwd["logprob"], wl.seed, sigma=0.3)
    ref = orc.lmhead_fused(h, W, wl.targets, old, tr_ref, a32, w32, np.float32(0.2), np.float32(0.2), 1.0)
    wl.token_rollout = tr
    out = run_fused(gh, wl, h, W, wl.targets, bwd=dict(old=old, adv=a32, weight=w32))
    assert out["err"] == 4                      # AERO_DERR_BAD_ROLLOUT
    gh.assert_loss(out["loss"].item(), ref["loss"], ref["loss_terms"])
    for k in ("logprob", "entropy", "lse"):
        assert np.abs(out[k].cpu().numpy().astype(np.float64) - fwd[k]).max() <= 2e-3, k
    dh = out["dhidden"].float().cpu().numpy().astype(np.float64)
    dw = out["dweight"].float().cpu().numpy().astype(np.float64)
    assert rowwise_close(dh, ref["dhidden"]) and rowwise_close(dw, ref["dweight"])
    assert not out["dhidden"].view(torch.int16)[[5, 6, 300]].any()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_fused_dweight_accumulates_over_micro_batches(gh, dtype):
    """AERO_DW_ACCUMULATE: two micro-batches (different tokens, the same weight) through one dweight buffer give
    the sum of their gradients.  fp32: exactly what adding the two separately computed results gives; bf16:
    the running value is rounded after each call, checked against the checker's sum to the row tolerance."""
    T, H, V = 520, 128, 3000
    wl1, h1, W = make(T, H, V, sigma_w=0.3)
    wl2, h2, _ = make(T, H, V, sigma_w=0.3, seed=11)

    def inputs(wl, h):
        ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, AdvParams())
        a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
        fwd = orc.lmhead_fused(h, W, wl.targets)
        old = ai.draw_old_logprob(fwd["logprob"], wl.seed, sigma=0.3)
        ref = orc.lmhead_fused(h, W, wl.targets, old, wl.token_rollout, a32, w32, np.float32(0.2), np.float32(0.2), 1.0)
        return dict(old=old, adv=a32, weight=w32), ref
    b1, ref1 = inputs(wl1, h1)
    b2, ref2 = inputs(wl2, h2)
    one = run_fused(gh, wl1, h1, W, wl1.targets, bwd=b1, dweight_dtype=dtype)
    two = run_fused(gh, wl2, h2, W, wl2.targets, bwd=b2, dweight_dtype=dtype)
    acc = one["dweight"].clone()
    both = run_fused(gh, wl2, h2, W, wl2.targets, bwd=b2, dweight_dtype=dtype, dw_into=acc)
    assert both["dweight"].data_ptr() == acc.data_ptr()
    if dtype == torch.float32:
        assert torch.equal(acc, one["dweight"] + two["dweight"])
    want = ref1["dweight"] + ref2["dweight"]
    assert rowwise_close(acc.float().cpu().numpy().astype(np.float64), want, frac=1e-2 if dtype == torch.float32 else 2e-2)
    assert rowwise_close(both["dhidden"].float().cpu().numpy().astype(np.float64), ref2["dhidden"])


def test_fused_matches_logits_path(gh):
    """Same inputs through the materialised-logits kernels: both routes agree with each other
    as closely as each agrees with the checker."""
    wl, h, W = make(512, 256, 8192, sigma_w=0.2)
    out = run_fused(gh, wl, h, W, wl.targets)
    z = (torch.from_numpy(h.view(np.int16)).to(gh.DEV).view(torch.bfloat16).float()
         @ torch.from_numpy(W.view(np.int16)).to(gh.DEV).view(torch.bfloat16).float().T).contiguous()
    lp, ent, lse, _ = gh.run_fwd(z, wl.T, wl.V, wl.V, wl.targets)
    assert (out["logprob"] - lp).abs().max().item() < 1e-3
    assert (out["entropy"] - ent).abs().max().item() < 1e-3


def test_fused_host_side_argument_errors(gh):
    """Status codes the fused call returns from host scalars alone; nothing is enqueued."""
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding
    T, H, V = 64, 64, 300
    dev = gh.DEV
    flat = torch.zeros(T * H + 8, dtype=torch.bfloat16, device=dev)
    w = torch.zeros((V, H), dtype=torch.bfloat16, device=dev)
    tg = torch.zeros(T, dtype=torch.int32, device=dev)
    lp, ent, lse = (torch.zeros(T, device=dev) for _ in range(3))
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=T, V=V, H=H), dtype=torch.uint8, device=dev)
    h_ok = flat[:T * H].view(T, H)
    h_off = flat[1:T * H + 1].view(T, H)          # 2 bytes past a 16-byte boundary
    assert h_off.data_ptr() % 16 == 2 and h_off.is_contiguous()
    aero.aero_lmhead_logprob_fused(h_ok, w, T, H, V, tg, lp, ent, lse, workspace=ws)
    with pytest.raises(aero.AeroError, match="pointer or leading dimension"):
        aero.aero_lmhead_logprob_fused(h_off, w, T, H, V, tg, lp, ent, lse, workspace=ws)
    with pytest.raises(aero.AeroError, match="workspace"):
        aero.aero_lmhead_logprob_fused(h_ok, w, T, H, V, tg, lp, ent, lse, workspace=ws[:1024])
    with pytest.raises(aero.AeroError, match="invalid size"):
        aero.aero_lmhead_logprob_fused(h_ok, w, T, 60, V, tg, lp, ent, lse, workspace=ws)       # H % 8 != 0
    with pytest.raises(aero.AeroError, match="NULL"):
        aero.aero_lmhead_logprob_fused(h_ok, w, T, H, V, None, lp, ent, lse, workspace=ws)
    # backward part: a dhidden that does not start on a 16-byte boundary
    R = 4
    old, adv, wr = torch.zeros(T, device=dev), torch.ones(R, device=dev), torch.ones(R, device=dev)
    tr = torch.zeros(T, dtype=torch.int32, device=dev)
    loss = torch.zeros(1, device=dev)
    dw = torch.zeros((V, H), device=dev)
    dflat = torch.zeros(T * H + 8, dtype=torch.bfloat16, device=dev)
    with pytest.raises(aero.AeroError, match="pointer or leading dimension"):
        aero.aero_lmhead_logprob_fused(h_ok, w, T, H, V, tg, lp, ent, lse, old, tr, adv, wr, R, loss=loss,
                                       dhidden=dflat[1:T * H + 1].view(T, H), dweight=dw, workspace=ws)
    aero.aero_lmhead_logprob_fused(h_ok, w, T, H, V, tg, lp, ent, lse, old, tr, adv, wr, R, loss=loss,
                                   dhidden=dflat[:T * H].view(T, H), dweight=dw, workspace=ws)
    torch.cuda.synchronize()
