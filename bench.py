#!/usr/bin/env python3
"""Throughput of the GRPO / AERO per-token hot path on one MI355X.

One step = one pass of the hot path over one synthetic micro-batch with inputs resident in
HBM: group advantages -> softmax statistics (log-prob, entropy, log-partition) -> clipped loss
+ gradient.  The headline workload is the Qwen2.5-Math-1.5B-shaped micro-batch (cfg2: 2 queries
x 8 rollouts x 1024 right-padded slots, V = 151936, bf16 logits).

Prints ONE JSON line.  Its top level is the headline workload: tokens/s (valid token rows per
second), the roofline of the dominant kernel measured with events on the launch stream, and the
float64 CPU checker timed on a bounded sample of the same workload as a baseline.  Under
"extra" the same process measures, each with its own roofline and CPU baseline: cfg2 with every
slot valid, cfg2 with its padding rows marked "leave the gradient row alone", the AERO-pruned
ragged batch (cfg3), the two LM-head-fused workloads (cfg4, cfg5), and one whole policy-update
step of 256 queries under plain grouping and under AERO's allocation + curation ("step": rollouts
and tokens trained on, time of both, CPU baseline; no roofline of its own, its calls are the cfg2 /
cfg3 kind).  `--workload X` measures X alone.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16

# HBM bytes per launch of the single-pass kernel on cfg2 from hardware counters (FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for an elementwise copy of known size;
# see profiles/logits_path_cfg2_hbm_traffic.txt).  Not a measurement of this run: a figure from
# that profile, valid only for the kernel sources it was taken on, so it is reported only while
# their hash still matches and is null otherwise.
MEASURED_TRAFFIC = {"cfg2": {"bytes": 7.8592e+09, "sources_sha256": "1f2a664388fee4d691d3d6e51fbeb08ae412c7b4a1b1344dbcf40e44b350189a"},
                    "cfg2-untouched": {"bytes": 5.7484e+09, "sources_sha256": "1f2a664388fee4d691d3d6e51fbeb08ae412c7b4a1b1344dbcf40e44b350189a"}}
TRAFFIC_SOURCES = ("paper_2602_14338_amd/csrc/grpo_single_pass.hip", "paper_2602_14338_amd/csrc/aero_device.h")
TRAFFIC_NOTE = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of the same kernel sources "
                "(profiles/logits_path_cfg2_hbm_traffic.txt), not of this run; null once the sources changed")


def measured_traffic(workload):
    import hashlib
    rec = MEASURED_TRAFFIC.get(workload)
    if rec is None:
        return None
    m = hashlib.sha256()
    for f in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, f), "rb") as fh:
            m.update(fh.read())
    return rec["bytes"] if m.hexdigest() == rec["sources_sha256"] else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None,
                    choices=["cfg1", "cfg2", "cfg2-dense", "cfg2-untouched", "cfg3", "cfg4", "cfg5", "step"],
                    help="measure this workload alone (default: cfg2 as the headline plus the extras)")
    ap.add_argument("--no-extras", action="store_true", help="headline workload only")
    ap.add_argument("--cpu-seconds", type=float, default=10.0,
                    help="CPU time budget of one workload's checker baseline (headline; extras get half)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gen-threads", type=int, default=16)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain elementwise copy kernel over the logits tensor (known size) before the timed "
                         "region, as the yardstick for hardware byte counters")
    ap.add_argument("--machine-ceilings", action="store_true",
                    help="instead of the benchmark, time plain library kernels on this GPU (an elementwise copy, a "
                         "fill, a reduction, a bf16 matmul of the LM-head shape) as context for the roofline fractions")
    return ap.parse_args()


def host_threads():
    """Threads the CPU baseline may use: the machine's CPU share (OMP_NUM_THREADS when set), never
    more than the cores that exist."""
    want = int(os.environ.get("OMP_NUM_THREADS", "16") or 16)
    return max(1, min(want, os.cpu_count() or 1))


def machine_ceilings(torch):
    """What plain vendor / framework kernels reach on this GPU, same footprints as the workloads.
    Context only: none of this is part of the library's path."""
    dev = "cuda:0"
    T, V, H = 16384, 151936, 1536
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    src = torch.randn((T // 4, V), device=dev, generator=gen).to(torch.bfloat16)
    src = src.repeat(4, 1)
    dst = torch.empty_like(src)

    def timed(fn, reps=10):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    nbytes = src.numel() * 2
    out = {"what": "plain library kernels on this GPU (context for roofline fractions)"}
    out["elementwise_copy_GBps"] = 2 * nbytes / timed(lambda: torch.neg(src, out=dst)) / 1e6
    out["fill_GBps"] = nbytes / timed(lambda: dst.zero_()) / 1e6
    out["row_max_read_GBps"] = nbytes / timed(lambda: torch.amax(src, dim=1)) / 1e6
    h = torch.randn((T, H), device=dev, generator=gen).to(torch.bfloat16)
    w = (torch.randn((V, H), device=dev, generator=gen) * 0.02).to(torch.bfloat16)
    ms = timed(lambda: torch.matmul(h, w.t()), reps=5)
    out["matmul_bf16_T16384_V151936_H1536_TFLOPs"] = 2.0 * T * V * H / ms / 1e9
    del src, dst
    h7 = torch.randn((T, 3584), device=dev, generator=gen).to(torch.bfloat16)
    w7 = (torch.randn((V, 3584), device=dev, generator=gen) * 0.02).to(torch.bfloat16)
    ms = timed(lambda: torch.matmul(h7, w7.t()), reps=3)
    out["matmul_bf16_T16384_V151936_H3584_TFLOPs"] = 2.0 * T * V * 3584 / ms / 1e9
    del h7, w7
    # The same contractions on all-zero operands: identical instruction stream and memory traffic, but no
    # bit toggles in the matrix pipes and on the data paths.  The gap to the Gaussian-operand figures is what
    # the power limit of this part costs (the clock it settles at under each load is in the counters).
    hz, wz = torch.zeros_like(h), torch.zeros_like(w)
    ms = timed(lambda: torch.matmul(hz, wz.t()), reps=5)
    out["matmul_bf16_T16384_V151936_H1536_zero_operands_TFLOPs"] = 2.0 * T * V * H / ms / 1e9
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding
    targets = torch.zeros(T, dtype=torch.int32, device=dev)
    lp, ent, lse = (torch.empty(T, device=dev) for _ in range(3))
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=T, V=V, H=H, R=1), dtype=torch.uint8, device=dev)
    for tag, hh, ww in (("gaussian", h, w), ("zero", hz, wz)):
        ms = timed(lambda: aero.aero_lmhead_logprob_fused(hh, ww, T, H, V, targets, lp, ent, lse, workspace=ws,
                                                          err_flag=err), reps=5)
        out["fused_forward_call_T16384_V151936_H1536_%s_operands_TFLOPs" % tag] = 2.0 * T * V * H / ms / 1e9
    print(json.dumps(out))


def median_ms(pairs):
    return float(np.median([a.elapsed_time(b) for a, b in pairs]))


# ----------------------------------------------------------------------------------------------
# logits path (cfg1, cfg2, cfg2-dense, cfg3)
# ----------------------------------------------------------------------------------------------

def cpu_baseline_logits(wl, host_old, budget_s):
    """The float64 checker as it stands (group advantages, forward statistics, loss + gradient) on
    valid rows drawn from evenly spaced 64-row blocks of the same batch: first on one thread, then
    with the rows shared out over a thread pool (numpy releases the GIL inside its row operations)."""
    import aero_inputs as ai
    from oracle import aero_oracle as orc
    T, V = wl.T, wl.V
    B = ai.workloads.ROWS_PER_BLOCK
    valid_mask = wl.token_rollout >= 0
    blocks = [b for b in range((T + B - 1) // B) if valid_mask[b * B:(b + 1) * B].any()]
    t0 = time.perf_counter()
    ga = orc.group_advantage(wl.rewards, wl.lengths, wl.group_offsets, wl.keep_priority, orc.AdvParams(**wl.adv_params))
    t_ga = time.perf_counter() - t0
    a32, w32 = ga["adv"].astype(np.float32), ga["weight"].astype(np.float32)
    eps = np.float32(wl.eps)

    def rows_of(block_ids):
        sel, parts = [], []
        for b in block_ids:
            r0, r1 = b * B, min(T, (b + 1) * B)
            m = valid_mask[r0:r1]
            sel.append(np.arange(r0, r1)[m])
            parts.append(wl.logits_rows(r0, r1)[m])           # input generation: untimed
        return np.concatenate(sel), np.concatenate(parts)

    def work(sel, hz):
        orc.logprob_fwd(hz, wl.dtype, V, wl.targets[sel])
        orc.grpo_loss_bwd(hz, wl.dtype, V, wl.targets[sel], host_old[sel], wl.token_rollout[sel], a32, w32, eps, eps, 1.0)

    # one thread: blocks until a third of the budget is spent
    order = np.random.default_rng(0).permutation(len(blocks))
    done1, t1, used = 0, 0.0, 0
    while used < len(order) and t1 < budget_s / 3:
        sel, hz = rows_of([blocks[order[used]]])
        used += 1
        t = time.perf_counter()
        work(sel, hz)
        t1 += time.perf_counter() - t
        done1 += len(sel)
    rate1 = done1 / t1
    # all cores: a sample sized for the rest of the budget at perfect scaling (at most 4096 rows), shared out in
    # pieces of 8 rows
    threads = host_threads()
    want = int(min(4096, max(threads * 8, rate1 * threads * budget_s * 2 / 3)))
    ids = []
    n = 0
    for j in order[::-1]:             # from the other end of the same random order
        if n >= want:
            break
        ids.append(blocks[j])
        n += int(valid_mask[blocks[j] * B:(blocks[j] + 1) * B].sum())
    sel, hz = rows_of(ids)
    pieces = [(sel[i:i + 8], hz[i:i + 8]) for i in range(0, len(sel), 8)]
    t = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda p: work(*p), pieces))
    tn = time.perf_counter() - t
    return {"value": len(sel) / (tn + t_ga), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "one_thread_value": done1 / (t1 + t_ga), "host_cpus_visible": os.cpu_count(),
            "sample": "valid token rows from randomly chosen 64-row blocks of the same workload, all three steps "
                      "(group advantages, statistics, loss + dlogits), numpy float64: %d rows on %d threads "
                      "(rows shared out over a thread pool) in %.1f s; %d rows on one thread in %.1f s"
                      % (len(sel), threads, tn, done1, t1)}


def run_logits(args, name, mods, headline):
    torch, ai, aero, binding = mods
    dev = "cuda:0"
    wl = ai.make_config("cfg2" if name in ("cfg2-dense", "cfg2-untouched") else name)
    if name == "cfg2-dense":   # same tensor shape, every slot a valid token
        wl.lengths[:] = wl.T // wl.R
        wl.token_rollout = np.repeat(np.arange(wl.R, dtype=np.int32), wl.T // wl.R)
    if name == "cfg2-untouched":   # padding rows marked "leave the gradient row alone" (a consumer that skips them)
        wl.token_rollout = np.where(wl.token_rollout < 0, binding.AERO_ROW_UNTOUCHED, wl.token_rollout).astype(np.int32)
    T, V, ld, R, Q = wl.T, wl.V, wl.ld, wl.R, wl.Q
    elt = 2 if wl.dtype == "bf16" else 4

    # ---- inputs -> HBM (untimed) ------------------------------------------------------
    t0 = time.time()
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    logits = torch.empty((T, ld), dtype=tdt, device=dev)
    chunk = 2048
    for r0 in range(0, T, chunk):
        r1 = min(T, r0 + chunk)
        h = wl.logits_rows(r0, r1, threads=args.gen_threads)
        src = torch.from_numpy(h.view(np.int16)).view(torch.bfloat16) if wl.dtype == "bf16" else torch.from_numpy(h)
        logits[r0:r1].copy_(src)
    gen_s = time.time() - t0

    def d(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    rewards, lengths, offsets = d(wl.rewards), d(wl.lengths), d(wl.group_offsets)
    keys = d(wl.keep_priority.view(np.int32))
    targets, token_rollout = d(wl.targets), d(wl.token_rollout)
    row_active = d((wl.token_rollout >= 0).astype(np.uint8))
    params = aero.AdvParams(**wl.adv_params)

    adv = torch.empty(R, device=dev)
    weight = torch.empty(R, device=dev)
    keep_mask = torch.empty(R, dtype=torch.uint8, device=dev)
    kept_index = torch.empty(R, dtype=torch.int32, device=dev)
    kept_offsets = torch.empty(Q + 1, dtype=torch.int32, device=dev)
    zero_var = torch.empty(Q, dtype=torch.uint8, device=dev)
    category = torch.empty(Q, dtype=torch.uint8, device=dev)
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    logprob = torch.empty(T, device=dev)
    entropy = torch.empty(T, device=dev)
    lse = torch.empty(T, device=dev)
    loss = torch.empty(1, device=dev)
    clip_frac = torch.empty(1, device=dev)
    lp_out = torch.empty(T, device=dev)
    dlogits = torch.empty_like(logits)
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_GRPO_LOSS_BWD, T=T, V=V, R=R), dtype=torch.uint8, device=dev)

    def step_adv():
        aero.aero_group_advantage(rewards, lengths, offsets, keys, Q, R, params, adv, weight, keep_mask,
                                  kept_index, kept_offsets, zero_var, category, err)

    def step_fwd():
        aero.aero_logprob_fwd(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err)

    def step_bwd():
        aero.aero_grpo_loss_bwd(logits, T, V, ld, targets, lse, old_logprob, token_rollout, adv, weight, R,
                                wl.eps, wl.eps, 1.0, loss, clip_frac, lp_out, dlogits, ws, err)

    def step_single():   # statistics, loss and dlogits in one pass over the logits
        aero.aero_grpo_loss_bwd(logits, T, V, ld, targets, None, old_logprob, token_rollout, adv, weight, R,
                                wl.eps, wl.eps, 1.0, loss, clip_frac, logprob, dlogits, ws, err,
                                entropy_out=entropy, lse_out=lse)

    # behaviour-policy log-probs: the current ones (from an untimed forward pass, as in
    # training where they come from an earlier pass of the same kernel) plus seeded noise
    step_adv()
    step_fwd()
    torch.cuda.synchronize()
    old_logprob = d(ai.draw_old_logprob(logprob.cpu().numpy(), wl.seed, sigma=0.05, eps_lo=wl.eps, eps_hi=wl.eps))

    if args.calibration_copy and headline:
        torch.neg(logits, out=dlogits)   # one elementwise kernel: reads and writes T*ld*elt bytes
    for _ in range(args.warmup):
        step_adv(); step_fwd(); step_bwd()
        step_adv(); step_single()
    torch.cuda.synchronize()
    K = args.steps

    # ---- forward call + loss call (6 bytes per logit), for comparison ---------------------
    K2 = K if headline else min(K, 20)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(K2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K2):
        ev[k][0].record(); step_adv()
        ev[k][1].record(); step_fwd()
        ev[k][2].record(); step_bwd()
        ev[k][3].record()
    torch.cuda.synchronize()
    wall2 = time.perf_counter() - t0
    ms_adv = median_ms([(e[0], e[1]) for e in ev])
    ms_fwd = median_ms([(e[1], e[2]) for e in ev])
    ms_bwd = median_ms([(e[2], e[3]) for e in ev])
    loss_two = loss.item()

    # ---- timed region: exactly K steps of the hot path (single pass over the logits) ------
    ev1 = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(K):
        step_adv()
        ev1[k][0].record(); step_single(); ev1[k][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_single = median_ms(ev1)
    assert int(err.item()) == 0 and np.isfinite(loss.item())
    assert abs(loss.item() - loss_two) <= 1e-5 * abs(loss_two) + 1e-12      # both routes give the same loss

    # ---- algorithmic bytes per launch ----------------------------------------------------
    n_valid = wl.n_valid
    adv_h = adv.cpu().numpy()
    trh = wl.token_rollout
    g_rows = int(((trh >= 0) & (adv_h[np.maximum(trh, 0)] != 0)).sum())   # rows that carry signal
    n_grad = int(round(g_rows * (1.0 - clip_frac.item())))   # unclipped rows: read + write
    n_written = T - int((trh == binding.AERO_ROW_UNTOUCHED).sum())   # rows whose gradient row is written at all
    n_zero = n_written - n_grad                          # write only
    row_bytes = V * elt
    fwd_bytes = n_valid * row_bytes
    bwd_bytes = n_grad * 2 * row_bytes + n_zero * row_bytes
    single_bytes = n_valid * row_bytes + n_written * row_bytes   # every valid row read once, every row written once
    valid_only_bytes = 2 * n_valid * row_bytes           # padding rows' zero fill not credited
    fwd_gbs = fwd_bytes / (ms_fwd * 1e-3) / 1e9
    bwd_gbs = bwd_bytes / (ms_bwd * 1e-3) / 1e9
    single_gbs = single_bytes / (ms_single * 1e-3) / 1e9
    valid_only_gbs = valid_only_bytes / (ms_single * 1e-3) / 1e9
    single_kernel = "k_row_stream" if V // 8 > 8 * 1024 else ("k_row_single_pass" if V >= 8192 else "k_logprob_fwd + k_dlogits")
    traffic = measured_traffic(name)
    out = {
        "metric": "tokens/s, GRPO logprob+loss fwd/bwd at V=%d" % V,
        "value": n_valid * K / wall,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "T_rows": T, "valid_tokens": n_valid, "V": V, "storage": wl.dtype,
                   "queries": Q, "rollouts": R, "signal_rows": g_rows, "grad_rows": n_grad,
                   "zero_fill_rows": n_zero, "clip_eps": wl.eps, "input_gen_s": round(gen_s, 1),
                   "step": "aero_group_advantage + aero_grpo_loss_bwd(lse=NULL, logprob/entropy/lse out)"},
        "kernels_ms": {"statistic": "median over the timed calls", "group_advantage": ms_adv,
                       "single_pass_loss_call": ms_single, "two_call_logprob_fwd": ms_fwd,
                       "two_call_grpo_loss_bwd": ms_bwd},
        "two_call_route": {"tokens_per_s": n_valid * K2 / wall2, "ms_per_step": wall2 / K2 * 1e3,
                           "logprob_fwd_GBps": fwd_gbs, "dlogits_GBps": bwd_gbs,
                           "logprob_fwd_frac": fwd_gbs / HBM_PEAK_GBS, "dlogits_frac": bwd_gbs / HBM_PEAK_GBS},
        "roofline": {"kernel": "%s (timed as the whole aero_grpo_loss_bwd call: counter preset + row order + the "
                               "row kernel + loss reduce; median of %d calls)" % (single_kernel, K),
                     "bound": "hbm", "achieved": single_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": single_gbs / HBM_PEAK_GBS, "algorithmic_bytes": single_bytes,
                     "accounting": "every valid row read once (2V bytes) + every row of the tensor written once "
                                   "(2V bytes; rows without gradient are zero-filled; rows marked untouched, which "
                                   "only cfg2-untouched has, are not written)",
                     "valid_rows_only": {"algorithmic_bytes": valid_only_bytes, "achieved": valid_only_gbs,
                                         "frac": valid_only_gbs / HBM_PEAK_GBS,
                                         "accounting": "4V bytes per valid row; the zero fill of padding rows is "
                                                       "not credited"},
                     "traffic": traffic, "traffic_source": TRAFFIC_NOTE if traffic is not None else None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_logits(wl, old_logprob.cpu().numpy(),
                                                  args.cpu_seconds if headline else args.cpu_seconds / 2)
    return out


# ----------------------------------------------------------------------------------------------
# one policy-update step through the logits path
# ----------------------------------------------------------------------------------------------

def bench_step(args, mods):
    """One policy-update step over 256 queries through the logits path, micro-batch by micro-batch,
    the paper's two ways (Sec. 4.1, Alg. 1, App. C budgets), over one rollout simulator (query q
    answers correctly with a latent probability p_q ~ Beta(1/2, 1/2)):
      grpo  16 rollouts per query, plain grouping, every rollout is packed and trained on;
      aero  the two-stage allocation loop on the host (8 exploration rollouts per query, rescue
            increments of 2, at most 10 iterations, at most 32 per query, at most 16 |P| in total)
            decides the ragged groups, the curation call applies Strategies 2 and 3 (posterior
            mean for all-equal groups, 1:1 rejection sampling), only kept rollouts are packed.
    Reports generated / trained rollouts and tokens per mode and the time of the curation call
    plus all loss / gradient calls.  One resident [mb_tokens, V] bf16 logits buffer serves every
    micro-batch (its content does not change the work done per row); the model forward / backward
    and rollout generation are outside this path."""
    torch, ai, aero, binding = mods
    from paper_2602_14338_amd import step
    from paper_2602_14338_amd.controller import allocate_rollouts
    dev = "cuda:0"
    V, mb_tokens, P, seed = 151936, 16384, 256, 5
    sim = ai.RolloutSimulator(seed, P, max_per_query=32, beta=0.5)
    wl = ai.make_config("cfg2")

    def d(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    logits = torch.empty((mb_tokens, V), dtype=torch.bfloat16, device=dev)
    for r0 in range(0, mb_tokens, 2048):
        h = wl.logits_rows(r0, r0 + 2048, threads=args.gen_threads)
        logits[r0:r0 + 2048].copy_(torch.from_numpy(h.view(np.int16)).view(torch.bfloat16))
    dlogits = torch.empty_like(logits)
    targets = d(wl.targets)
    lp, lse = torch.empty(mb_tokens, device=dev), torch.empty(mb_tokens, device=dev)
    aero.aero_logprob_fwd(logits, mb_tokens, V, V, targets, None, lp, None, lse)
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    old = (lp + 0.05 * torch.randn(mb_tokens, device=dev, generator=g)).contiguous()

    # the two sets of groups (host work of the sampler, untimed)
    drawn = [sim.draw(q, 0, 16) for q in range(P)]
    plain = dict(rewards=np.concatenate([r for r, _ in drawn]), lengths=np.concatenate([l for _, l in drawn]),
                 offsets=np.arange(0, 16 * P + 1, 16, dtype=np.int32), generated=16 * P)
    alloc = allocate_rollouts(sim.draw, P, n_explore=8, n_extra=2, k_max=10, n_max=32, n_budget=16, S=0)
    curated = dict(rewards=alloc.rewards, lengths=alloc.lengths, offsets=alloc.group_offsets, generated=alloc.generated)
    out = {}
    for mode, grp, params in (("grpo", plain, dict()), ("aero", curated, dict(reject_enable=1, posterior_mode=1))):
        R = grp["rewards"].size
        rewards, lengths, offsets = d(grp["rewards"]), d(grp["lengths"]), d(grp["offsets"])
        keys = d(np.random.default_rng(seed).integers(0, 2 ** 32, size=R, dtype=np.uint32).view(np.int32))
        p = aero.AdvParams(**params)
        cur = step.curate(rewards, lengths, offsets, keys, p)
        torch.cuda.synchronize()
        assert int(cur.err.item()) == 0
        keep = cur.keep_mask.cpu().numpy()
        rollouts = np.nonzero(keep)[0]
        plan = step.plan_microbatches(grp["lengths"], rollouts, mb_tokens)   # data-loader work, untimed
        plan_d = d(plan)
        signal = (cur.adv.cpu().numpy()[rollouts] != 0) & (cur.weight.cpu().numpy()[rollouts] != 0)

        def run():
            c = step.curate(rewards, lengths, offsets, keys, p)
            return step.loss_bwd_microbatches(plan_d, lambda k: logits, lambda k: targets, lambda k: old,
                                              lambda k: dlogits, c.adv, c.weight, V, V, 0.2, 0.2)
        run()
        torch.cuda.synchronize()
        times = []
        for _ in range(3):
            t0 = time.perf_counter()
            losses = run()
            torch.cuda.synchronize()
            times.append((time.perf_counter() - t0) * 1e3)
        out[mode] = {"rollouts_generated": int(grp["generated"]), "rollouts_generated_per_query": grp["generated"] / P,
                     "rollouts_trained": int(rollouts.size), "rollouts_trained_per_query": rollouts.size / P,
                     "tokens_generated": int(grp["lengths"].sum()),
                     "tokens_trained": int(grp["lengths"][rollouts].sum()),
                     "tokens_with_signal": int(grp["lengths"][rollouts][signal].sum()),
                     "zero_variance_groups": int(cur.zero_var.sum().item()),
                     "micro_batches": int(plan.shape[0]), "ms": float(np.median(times)),
                     "loss": float(losses.double().sum().item())}
    out["aero"]["rescue"] = {"queries_rescued": int((alloc.rescued_at > 0).sum()),
                             "queries_never_rescued": int((alloc.rescued_at < 0).sum()),
                             "iterations": int(alloc.iterations)}
    res = {
        "metric": "ms per policy-update step on the logits path (256 queries, V=151936), AERO allocation + curation",
        "value": out["aero"]["ms"], "unit": "ms", "n_gpus": 1, "steps": 3, "warmup": 1,
        "ms_per_step": out["aero"]["ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "step", "queries": P, "micro_batch_rows": mb_tokens, "V": V, "storage": "bf16",
                   "simulator": "p_q ~ Beta(0.5, 0.5), lengths U{128..2048}", "n_explore": 8, "n_extra": 2,
                   "k_max": 10, "n_max": 32, "n_budget": 16, "S": 0, "k_ratio": 1},
        "grpo": out["grpo"], "aero": out["aero"],
        "trained_token_ratio_aero_over_grpo": out["aero"]["tokens_trained"] / out["grpo"]["tokens_trained"],
        "time_ratio_aero_over_grpo": out["aero"]["ms"] / out["grpo"]["ms"],
        "paper_context": "the paper reports about 4.6 trained rollouts per query of 16 and 45-48 % less time / "
                         "compute for the whole training step on other hardware (Sec. 4.4, Table 1); this line "
                         "covers the loss / gradient path only",
    }
    if not args.no_cpu_baseline:
        base = cpu_baseline_logits(wl, old.cpu().numpy(), args.cpu_seconds / 2)
        rate = base["value"]
        res["cpu_baseline"] = {"value": out["aero"]["tokens_trained"] / rate * 1e3, "unit": "ms", "cores": base["cores"],
                               "kind": "oracle",
                               "sample": "the aero step's trained tokens at the checker's per-row rate (%.0f tokens/s; %s)"
                                         % (rate, base["sample"])}
    return res


# ----------------------------------------------------------------------------------------------
# fused LM-head path (cfg4, cfg5)
# ----------------------------------------------------------------------------------------------

def cpu_baseline_fused(wl, h_rows, W_bits, host_old, a32, w32, budget_s):
    """The float64 checker's fused definition (float64 product h W^T through the BLAS dgemm numpy
    links, then statistics, loss, dz, dhidden = dz W and dweight = dz^T h) on a sample of token
    rows of the same batch against the full weight matrix: with the BLAS's threads, then with one."""
    from oracle import aero_oracle as orc
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([int(i.get("num_threads", 1)) for i in threadpool_info() if i.get("user_api") == "blas"] or [1])
    except Exception:   # no control over the BLAS pool: report what it is given
        threadpool_limits, blas_threads = None, host_threads()
    T = wl.T
    valid = np.nonzero(wl.token_rollout >= 0)[0]
    eps = np.float32(wl.eps)
    flop_per_row = 8.0 * wl.V * wl.H
    # sample sizes from a nominal dgemm rate (20 GFLOP/s per thread), the conversions of W included in the time
    n_all = int(np.clip(budget_s * 0.45 * 20e9 * blas_threads / flop_per_row, 16, 512))
    n_one = int(np.clip(budget_s * 0.25 * 20e9 / flop_per_row, 4, 64))

    def run(n):
        sel = valid[np.linspace(0, len(valid) - 1, n).astype(np.int64)]
        t = time.perf_counter()
        orc.lmhead_fused(h_rows(sel), W_bits, wl.targets[sel], host_old[sel], wl.token_rollout[sel], a32, w32,
                         eps, eps, 1.0)
        return n, time.perf_counter() - t

    n_a, t_a = run(n_all)
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            n_1, t_1 = run(n_one)
    else:
        n_1, t_1 = n_a, t_a
    return {"value": n_a / t_a, "unit": "tokens/s", "cores": blas_threads, "kind": "oracle",
            "one_thread_value": n_1 / t_1, "host_cpus_visible": os.cpu_count(),
            "sample": "%d evenly spaced valid token rows of the same workload against the full [V, H] weight, the "
                      "checker's fused definition (float64 product, statistics, loss, dz, dhidden, dweight), numpy "
                      "float64 with %d BLAS threads in %.1f s; %d rows with one thread in %.1f s (each run also "
                      "widens the whole weight matrix to float64, as the checker does)"
                      % (n_a, blas_threads, t_a, n_1, t_1)}


def run_fused(args, name, mods):
    """Fused LM-head workloads: one step = group advantages + fused forward + loss + dhidden/dweight."""
    torch, ai, aero, binding = mods
    dev = "cuda:0"
    wl = ai.make_config(name)
    T, H, V, R, Q = wl.T, wl.H, wl.V, wl.R, wl.Q
    t0 = time.time()
    W_bits = wl.weight_rows(0, V, threads=args.gen_threads)

    def up_rows(gen, n, width):
        out = torch.empty((n, width), dtype=torch.bfloat16, device=dev)
        for r0 in range(0, n, 8192):
            r1 = min(n, r0 + 8192)
            out[r0:r1].copy_(torch.from_numpy(gen(r0, r1, threads=args.gen_threads).view(np.int16)).view(torch.bfloat16))
        return out

    hidden = up_rows(wl.hidden_rows, T, H)
    weight = torch.from_numpy(W_bits.view(np.int16)).to(dev).view(torch.bfloat16)
    gen_s = time.time() - t0

    def d(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(dev)

    rewards, lengths, offsets = d(wl.rewards), d(wl.lengths), d(wl.group_offsets)
    keys = d(wl.keep_priority.view(np.int32))
    targets, token_rollout = d(wl.targets), d(wl.token_rollout)
    params = aero.AdvParams(**wl.adv_params)
    adv, wgt = torch.empty(R, device=dev), torch.empty(R, device=dev)
    keep_mask = torch.empty(R, dtype=torch.uint8, device=dev)
    kept_index = torch.empty(R, dtype=torch.int32, device=dev)
    kept_offsets = torch.empty(Q + 1, dtype=torch.int32, device=dev)
    zero_var = torch.empty(Q, dtype=torch.uint8, device=dev)
    category = torch.empty(Q, dtype=torch.uint8, device=dev)
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    lp, ent, lse = (torch.empty(T, device=dev) for _ in range(3))
    loss, clip = torch.empty(1, device=dev), torch.empty(1, device=dev)
    dh = torch.empty((T, H), dtype=torch.bfloat16, device=dev)
    dw = torch.empty((V, H), dtype=torch.bfloat16, device=dev)
    ws = torch.empty(aero.aero_workspace_bytes(binding.OP_LMHEAD_FUSED, T=T, V=V, H=H, R=R), dtype=torch.uint8,
                     device=dev)

    def step_adv():
        aero.aero_group_advantage(rewards, lengths, offsets, keys, Q, R, params, adv, wgt, keep_mask, kept_index,
                                  kept_offsets, zero_var, category, err)

    def step_fwd_only():
        aero.aero_lmhead_logprob_fused(hidden, weight, T, H, V, targets, lp, ent, lse, workspace=ws, err_flag=err)

    def step_full():
        aero.aero_lmhead_logprob_fused(hidden, weight, T, H, V, targets, lp, ent, lse, old_lp, token_rollout, adv,
                                       wgt, R, wl.eps, wl.eps, 1.0, loss, clip, dh, dw, ws, err)

    step_adv()
    step_fwd_only()
    torch.cuda.synchronize()
    host_old = ai.draw_old_logprob(lp.cpu().numpy(), wl.seed, sigma=0.05, eps_lo=wl.eps, eps_hi=wl.eps)
    old_lp = d(host_old)
    K = max(1, min(args.steps, 20 if H <= 2048 else 10))
    W = max(1, min(args.warmup, 5 if H <= 2048 else 3))
    for _ in range(W):
        step_adv(); step_full()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K)]
    t0 = time.perf_counter()
    for k in range(K):
        step_adv()
        ev[k][0].record(); step_full(); ev[k][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_fused = median_ms(ev)
    # forward alone, for the split
    ef = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(max(3, K // 2))]
    for a, b in ef:
        a.record(); step_fwd_only(); b.record()
    torch.cuda.synchronize()
    ms_fwd = median_ms(ef)
    assert int(err.item()) == 0 and np.isfinite(loss.item())

    adv_h, wgt_h = adv.cpu().numpy(), wgt.cpu().numpy()
    tr = wl.token_rollout
    signal = int(((tr >= 0) & (adv_h[np.maximum(tr, 0)] != 0)).sum())
    n_grad = int(round(signal * (1.0 - clip.item())))
    flops = 2.0 * wl.n_valid * V * H + 6.0 * n_grad * V * H
    tf = flops / (ms_fused * 1e-3) / 1e12
    # what the kernels execute: the backward pass reuses the exponentials the forward pass stored for the rows
    # that may carry gradient (signal rows) instead of forming their logits again, so its contractions are two
    flops_exec = 2.0 * wl.n_valid * V * H + 4.0 * signal * V * H
    tf_exec = flops_exec / (ms_fused * 1e-3) / 1e12
    tf_fwd = 2.0 * wl.n_valid * V * H / (ms_fwd * 1e-3) / 1e12
    out = {
        "metric": "tokens/s, fused LM-head GRPO logprob+loss fwd/bwd at V=%d, H=%d" % (V, H),
        "value": wl.n_valid * K / wall, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "T": T, "valid_tokens": wl.n_valid, "H": H, "V": V, "queries": Q, "rollouts": R,
                   "signal_rows": signal, "grad_rows": n_grad, "input_gen_s": round(gen_s, 1),
                   "step": "aero_group_advantage + aero_lmhead_logprob_fused (forward + loss + dhidden + dweight)"},
        "kernels_ms": {"statistic": "median over the timed calls", "fused_fwd_bwd_call": ms_fused,
                       "fused_fwd_only_call": ms_fwd},
        "roofline": {"kernel": "whole aero_lmhead_logprob_fused call (fwd + bwd; median of %d calls), algorithmic flops "
                               "2 T_valid V H + 6 T_grad V H" % K, "bound": "mfma", "achieved": tf,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_BF16_PEAK_TFLOPS,
                     "algorithmic_flops": flops,
                     "accounting": "forward on every row with a target (2 V H per row) + recompute, dhidden and dweight "
                                   "on the rows with gradient (6 V H per row): the method's count, whatever the kernels do",
                     "executed": {"flops": flops_exec, "achieved": tf_exec, "frac": tf_exec / MFMA_BF16_PEAK_TFLOPS,
                                  "accounting": "2 V H per row with a target + 4 V H per signal row: the logits of the "
                                                "gradient rows are not formed a second time (the forward pass leaves "
                                                "exp(z - z_y) for them), so the recompute term is credited above but "
                                                "not executed"},
                     "traffic": None},
        "roofline_fwd": {"kernel": "fused forward call (gather + k_fused_stats + combine), 2 T_valid V H", "bound": "mfma",
                         "achieved": tf_fwd, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf_fwd / MFMA_BF16_PEAK_TFLOPS, "traffic": None},
    }
    if not args.no_cpu_baseline:
        del dw, dh, ws
        out["cpu_baseline"] = cpu_baseline_fused(wl, lambda sel: np.stack([wl.hidden_rows(int(t), int(t) + 1)[0] for t in sel]),
                                                 W_bits, host_old, adv_h.astype(np.float32), wgt_h.astype(np.float32),
                                                 args.cpu_seconds / 2)
    return out


def run_workload(args, name, mods, headline):
    if name in ("cfg4", "cfg5"):
        return run_fused(args, name, mods)
    if name == "step":
        return bench_step(args, mods)
    return run_logits(args, name, mods, headline)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this library runs on ONE GPU only (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import aero_inputs as ai
    import paper_2602_14338_amd as aero
    from paper_2602_14338_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    mods = (torch, ai, aero, binding)

    if args.machine_ceilings:
        return machine_ceilings(torch)
    if args.workload is not None:
        print(json.dumps(run_workload(args, args.workload, mods, headline=True)))
        return
    out = run_workload(args, "cfg2", mods, headline=True)
    if not args.no_extras:
        out["extra"] = {}
        for name in ("cfg2-dense", "cfg2-untouched", "cfg3", "cfg4", "cfg5", "step"):
            torch.cuda.empty_cache()
            t0 = time.time()
            res = run_workload(args, name, mods, headline=False)
            res["bench_wall_s"] = round(time.time() - t0, 1)
            out["extra"][name] = res
            print("bench.py: %s done in %.1f s" % (name, res["bench_wall_s"]), file=sys.stderr, flush=True)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
