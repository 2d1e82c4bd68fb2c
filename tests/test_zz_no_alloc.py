"""The loss entry point that owns its scratch (`aero_grpo_loss_bwd_noalloc`, for callers that
cannot allocate device memory) against the workspace-taking `aero_grpo_loss_bwd` on the same
inputs: same kernels, so every output must agree bit for bit.  Two calls in a row share the
library's one scratch array on this GPU; the second has fewer rows, so anything the first call
left behind there would show.  Both routes are covered: statistics given (two-call route) and
statistics computed inside (one pass over the logits, streaming kernel at V = 151936).
"""
import numpy as np
import pytest
import torch

import aero_inputs as ai

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gh():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_helpers
    return gpu_helpers


def both_entry_points(gh, wl, single_pass, entropy_coef=0.0):
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding
    T, V, ld, R, Q = wl.T, wl.V, wl.ld, wl.R, wl.Q
    dev = gh.DEV
    logits = gh.logits_to_dev(wl.logits_rows(0, T), wl.dtype)
    targets, tr = gh.dev(wl.targets), gh.dev(wl.token_rollout)
    # curation and forward statistics from the library itself: this test compares two entry
    # points of the library with each other, the checker is not involved
    adv, weight = torch.empty(R, device=dev), torch.empty(R, device=dev)
    scratch_outs = [torch.empty(R, dtype=torch.uint8, device=dev), torch.empty(R, dtype=torch.int32, device=dev),
                    torch.empty(Q + 1, dtype=torch.int32, device=dev), torch.empty(Q, dtype=torch.uint8, device=dev),
                    torch.empty(Q, dtype=torch.uint8, device=dev)]
    aero.aero_group_advantage(gh.dev(wl.rewards), gh.dev(wl.lengths), gh.dev(wl.group_offsets), None, Q, R,
                              aero.AdvParams(), adv, weight, *scratch_outs)
    lp, ent, lse = (torch.empty(T, device=dev) for _ in range(3))
    aero.aero_logprob_fwd(logits, T, V, ld, targets, None, lp, ent, lse)
    torch.cuda.synchronize()
    noise = np.random.default_rng(wl.seed + 5).normal(0, 0.3, size=T).astype(np.float32)
    old = (lp + gh.dev(noise)).contiguous()

    def outputs():
        return dict(loss=torch.full((1,), 7.0, device=dev), clip=torch.full((1,), 7.0, device=dev),
                    lp=torch.full((T,), 7.0, device=dev), dz=torch.full_like(logits, 7.0),
                    err=torch.zeros(1, dtype=torch.int32, device=dev),
                    ent=torch.full((T,), 7.0, device=dev) if single_pass else None,
                    lse=torch.full((T,), 7.0, device=dev) if single_pass else None)

    a, b = outputs(), outputs()
    common = dict(entropy_coef=entropy_coef, entropy=None if single_pass else ent)
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_GRPO_LOSS_BWD, T=T, V=V, R=R), dtype=torch.uint8, device=dev)
    aero.aero_grpo_loss_bwd(logits, T, V, ld, targets, None if single_pass else lse, old, tr, adv, weight, R,
                            0.2, 0.2, 1.0, a["loss"], a["clip"], a["lp"], a["dz"], ws, a["err"],
                            entropy_out=a["ent"], lse_out=a["lse"], **common)
    aero.aero_grpo_loss_bwd_noalloc(logits, T, V, ld, targets, None if single_pass else lse, old, tr, adv, weight, R,
                                    0.2, 0.2, 1.0, b["loss"], b["clip"], b["lp"], b["dz"], b["err"],
                                    entropy_out=b["ent"], lse_out=b["lse"], **common)
    torch.cuda.synchronize()
    assert int(a["err"].item()) == 0 and int(b["err"].item()) == 0
    assert np.isfinite(a["loss"].item()) and a["loss"].item() != 7.0
    assert 0.0 < a["clip"].item() < 1.0                      # both clip branches present
    assert (a["dz"].view(torch.int16) != 0).any()
    for k in a:
        if a[k] is None or k == "err":
            continue
        x, y = a[k], b[k]
        bits = torch.int16 if x.dtype == torch.bfloat16 else torch.int32
        assert torch.equal(x.view(bits), y.view(bits)), k


@pytest.mark.parametrize("single_pass", [False, True])
def test_noalloc_matches_workspace_entry_point_twice(gh, single_pass):
    # 320 rows: more than one row per persistent workgroup in the streaming kernel; then 96
    big = ai.make_config("cfg3", V=151936, T=320, Q=64, len_lo=1, len_hi=12)
    small = ai.make_config("cfg2", V=151936, slots=6, len_lo=1, len_hi=6)
    assert small.T < big.T
    both_entry_points(gh, big, single_pass)
    both_entry_points(gh, small, single_pass, entropy_coef=1e-3)


def test_noalloc_rejects_sizes_beyond_its_capacity(gh):
    import paper_2602_14338_amd as aero
    z = torch.zeros((4, 16), dtype=torch.bfloat16, device=gh.DEV)
    t = torch.zeros(4, dtype=torch.int32, device=gh.DEV)
    f = torch.zeros(4, device=gh.DEV)
    with pytest.raises(aero.AeroError, match="capacity"):
        aero.aero_grpo_loss_bwd_noalloc(z, 65537, 16, 16, t, None, f, t, f, f, 4, 0.2, 0.2, 1.0, f[:1], None, None, None)
