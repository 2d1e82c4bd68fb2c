/*
 * aero.h - C ABI of the GPU library for the per-token hot path of a group-based RL update
 * (GRPO with AERO's curated rollout groups), written for AMD MI355X (gfx950).
 *
 * Conventions (all entry points)
 *   - Every array pointer is a DEVICE pointer owned by the caller.  The library never
 *     allocates or frees device memory; scratch comes from the caller's `workspace` (size it
 *     with aero_workspace_bytes; 256-byte aligned).  The one exception is stated at
 *     aero_grpo_loss_bwd_noalloc, which uses a fixed array inside the library instead.
 *   - Scalars, the parameter struct and the returned status live on the HOST.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and the call returns without synchronising.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - Outputs are fully overwritten (one exception, on request: dlogits rows of token rows marked
 *     AERO_ROW_UNTOUCHED).  Nullable arguments are marked.
 *   - Shape errors that can be seen from host scalars return a status code and enqueue
 *     nothing.  Errors that depend on device data never fault; a bit is OR-ed into the
 *     optional device word `err_flag`, which the caller zeroes:
 *       a sampled-token id >= V or a rollout index >= R: the token row is treated as ignored;
 *       a reward other than 0 or 1 where binary ones are required: the group is still
 *       processed, with every reward other than exactly 1 counted as incorrect.
 *   - "Ignored row": a token row with a negative sampled-token id, a negative rollout
 *     index, or row_active == 0.  It is not read, its outputs are 0 (gradient rows +0, or left as
 *     they are when the rollout index is AERO_ROW_UNTOUCHED), and nothing about it is flagged,
 *     whatever its other fields hold.
 *   - Logits (and hidden states / weights) must be finite.  An infinite or NaN logit gives NaN
 *     statistics for its row (the entropy term contains 0 * inf); vocabulary masking with -inf
 *     is not part of the policy the paper defines (App. C).
 */
#ifndef AERO_H
#define AERO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t aero_status;
enum {
  AERO_OK = 0,
  AERO_ERR_NULL = 1,       /* a required pointer is NULL */
  AERO_ERR_SHAPE = 2,      /* negative size, ld < V, V or H outside the supported range */
  AERO_ERR_DTYPE = 3,      /* dtype code not supported by this call */
  AERO_ERR_ALIGN = 4,      /* pointer or leading dimension violates a stated alignment */
  AERO_ERR_WORKSPACE = 5,  /* workspace NULL, misaligned or smaller than aero_workspace_bytes */
  AERO_ERR_HIP = 6,        /* a HIP launch failed; hipGetLastError has the detail */
  AERO_ERR_LIMIT = 7       /* size beyond the fixed capacity of an entry point that owns its scratch */
};

/* Storage types of logits / dlogits.  AERO_F16 (IEEE binary16) and AERO_F8E4M3 are accepted by
 * aero_logprob_fwd and aero_grpo_loss_bwd only.  fp16 gradient entries round to the fp16 grid (subnormals
 * below 6.1e-5, zero below 3e-8): pass a grad_scale that lifts them, as with any fp16 gradient.
 * AERO_F8E4M3 is the 8-bit float with 4 exponent bits (bias 7) and 3 mantissa bits in the variant without
 * infinities (sign.1111.111 is NaN, largest finite value 448, subnormals are multiples of 2^-9); gradient
 * entries are rounded to nearest even on that grid and saturate at +-448, so a grad_scale is needed all the
 * more.  All arithmetic is fp32 whatever the storage type. */
enum { AERO_F32 = 0, AERO_BF16 = 1, AERO_F16 = 2, AERO_F8E4M3 = 3 };

/* OR-ed into the dweight_dtype argument of aero_lmhead_logprob_fused: dweight += dz^T hidden instead of
 * dweight = ..., i.e. the caller's buffer accumulates the gradient over the micro-batches of a step (the sum is
 * formed in fp32 per entry; with a bf16 buffer the running value is rounded after every call). */
enum { AERO_DW_ACCUMULATE = 0x100 };

/* token_rollout[t] of a token row that belongs to no rollout.  Both are ignored rows; AERO_ROW_UNTOUCHED
 * additionally tells aero_grpo_loss_bwd (and its _noalloc form) not to write the row's dlogits at all, for
 * callers whose consumer of the gradient skips padding rows or who keep those rows zero themselves.  Any other
 * negative value means AERO_ROW_PADDING. */
enum { AERO_ROW_PADDING = -1, AERO_ROW_UNTOUCHED = -2 };

/* bits of the device error word */
enum { AERO_DERR_NONBINARY_REWARD = 1, AERO_DERR_BAD_TARGET = 2, AERO_DERR_BAD_ROLLOUT = 4 };

/* group_category[q]: low two bits = four-way category by success rate u = c/n with
 * threshold tau (App. C, "Problem Categorization"); bit 2 = rescue stratum u <= S/n
 * (Sec. 4.2 Strategy 1, Alg. 1). */
enum { AERO_CAT_ZERO = 0, AERO_CAT_PARTIAL = 1, AERO_CAT_GOOD = 2, AERO_CAT_PERFECT = 3,
       AERO_CAT_RESCUE_BIT = 4 };

enum { AERO_OP_GROUP_ADVANTAGE = 0, AERO_OP_LOGPROB_FWD = 1, AERO_OP_GRPO_LOSS_BWD = 2,
       AERO_OP_LMHEAD_FUSED = 3 };

/* Hyper-parameters of the curation step (Table 8; Sec. 4.2). */
typedef struct {
  int32_t k_ratio;         /* Strategy 3: keep m = k*c incorrect rollouts, k >= 1 (paper: 1)      */
  int32_t s_rescue;        /* Strategy 1: rescue threshold S on the number of correct rollouts (0) */
  int32_t tau_num, tau_den;/* tau = tau_num/tau_den (1/2): u < tau is "partial", else "good"       */
  int32_t zero_keep;       /* Strategy 2: rollouts kept from an all-equal group (4)                */
  int32_t reject_enable;   /* 0 = plain GRPO grouping: every rollout is kept                       */
  int32_t posterior_mode;  /* 0 = all-equal groups get advantage 0; 1 = Beta posterior mean        */
  float alpha0, beta0;     /* Beta prior (1, 1)                                                    */
} aero_adv_params;

const char* aero_status_string(aero_status s);

/* Bytes of workspace the given call needs for these sizes (0 if it needs none).
 * Sizes that do not apply to an op are ignored. */
size_t aero_workspace_bytes(int32_t op, int64_t T, int32_t V, int32_t H, int32_t R, int32_t Q);

/*
 * Group statistics, kept subset, group-relative advantages and per-rollout loss weights.
 *
 * Defines: Eq. 1 (advantage = (r - mean) / std over the group, population std, no epsilon);
 * Sec. 3.2 (all rewards equal => advantage 0); Sec. 4.1 / Alg. 1 and App. C (strata);
 * Sec. 4.2 Strategy 2 (posterior mean u~ = (c + alpha0)/(n + alpha0 + beta0) replaces the
 * mean of all-fail / all-correct groups, zero_keep rollouts kept) and Strategy 3 (partial
 * groups keep all c correct rollouts and m = min(k c, n - c) incorrect ones); Theorem 4.1
 * (statistics are taken over the kept subset); Eq. 2 (weights 1/N and 1/|o_i|).
 *
 * Inputs   rewards[R] f32 (must be exactly 0 or 1 when reject_enable or posterior_mode is
 *          set), lengths[R] i32 (|o_i|, full valid response length), group_offsets[Q+1] i32
 *          (CSR, ascending, off[0] = 0, off[Q] = R, group q = rollouts [off[q], off[q+1]); every rollout
 *          belongs to exactly one group: a rollout outside all groups would be left unwritten), keep_priority[R] u32 or
 *          NULL (down-sampling keeps the smallest (key, index) pairs; NULL = index order).
 * Outputs  adv[R] f32, weight[R] f32 (1/(Q * kept_q * lengths[i]) for kept rollouts, else 0),
 *          keep_mask[R] u8, kept_index[R] i32 (first kept_offsets[Q] entries: kept rollout
 *          indices, ascending), kept_offsets[Q+1] i32 (CSR of kept counts),
 *          group_zero_var[Q] u8 (kept rewards all equal, or nothing kept),
 *          group_category[Q] u8 (AERO_CAT_*).
 * In posterior mode the advantage of an all-equal group is (r - u~)/sqrt(u~(1-u~)).
 * Q = 0 or R = 0 is valid.  p is a host pointer, read before the call returns.
 */
aero_status aero_group_advantage(
    const float* rewards, const int32_t* lengths, const int32_t* group_offsets,
    const uint32_t* keep_priority /*nullable*/, int32_t Q, int32_t R,
    const aero_adv_params* p,
    float* adv, float* weight, uint8_t* keep_mask, int32_t* kept_index, int32_t* kept_offsets,
    uint8_t* group_zero_var, uint8_t* group_category,
    int32_t* err_flag /*nullable*/, void* stream);

/*
 * Softmax policy statistics per token row (App. C: pi = softmax(f_theta); Sec. D: the
 * log-prob of the sampled token is what the update consumes; Table 8: an entropy term is used).
 *   lse[t] = log sum_j exp z[t,j],  logprob[t] = z[t, targets[t]] - lse[t],
 *   entropy[t] = lse[t] - sum_j softmax(z[t])_j z[t,j]          (natural log, temperature 1)
 *
 * logits   [T, ld] row-major, dtype AERO_BF16, AERO_F16, AERO_F8E4M3 or AERO_F32, ld >= V; columns >= V are never
 *          read.  Any alignment works; rows whose base and ld*sizeof(elt) are multiples of
 *          16 bytes take the 128-bit load path.
 * targets  i32[T] sampled-token ids; row_active u8[T] or NULL.
 * Outputs  logprob[T], lse[T] f32; entropy[T] f32 or NULL.  Ignored rows get 0.
 * Accumulation is fp32.  T = 0 is valid.  1 <= V <= 2^24.
 */
aero_status aero_logprob_fwd(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
    const int32_t* targets, const uint8_t* row_active /*nullable*/,
    float* logprob, float* entropy /*nullable*/, float* lse,
    int32_t* err_flag /*nullable*/, void* stream);

/*
 * Clipped-ratio surrogate loss (Eq. 2 with beta = 0, sign flipped: loss = -J) and its
 * gradient with respect to the logits (App. A.1).
 *   token t of rollout i = token_rollout[t] with A = adv[i] != 0 and w = weight[i] != 0:
 *     rho = exp(logprob[t] - old_logprob[t])
 *     loss -= w * min(rho A, clip(rho, 1 - eps_lo, 1 + eps_hi) A)
 *     g_t  = -grad_scale * w * A * rho   if the unclipped branch is active
 *            (A > 0: rho <= 1 + eps_hi;  A < 0: rho >= 1 - eps_lo), else 0
 *     dlogits[t, j] = g_t * (1[j == targets[t]] - exp(z[t,j] - lse[t]))
 *   every other row (padding, ignored, A == 0, w == 0, clipped): dlogits row = +0, except rows with
 *   token_rollout[t] == AERO_ROW_UNTOUCHED, whose dlogits row is neither read nor written (their
 *   scalar outputs are 0 like those of any ignored row).
 * Entropy bonus (Table 8 lists a coefficient; it is aggregated with Eq. 2's weights): with
 * entropy_coef = c != 0 every token of a rollout with w != 0, whatever A or the clip decision,
 *     loss -= c * w * H_t,   dlogits[t, j] += grad_scale * c * w * p_j * (ln p_j + H_t),
 *     p_j = exp(z[t,j] - lse[t]), H_t = entropy of row t.
 * KL penalty (the - beta D_KL(pi || pi_ref) term of Eq. 2; the paper names no estimator, the
 * per-token one of the GRPO literature is used): with kl_coef = beta != 0 every token of a rollout
 * with w != 0, clipped or not,
 *     d = ref_logprob[t] - logprob[t],  loss += beta * w * (exp(d) - d - 1),
 *     g_t += grad_scale * beta * w * (1 - exp(d)).
 *
 * logits / dlogits  [T, ld], same dtype and ld; dlogits may alias logits (in place).
 * lse      f32[T] from aero_logprob_fwd, or NULL: then the statistics are computed here.  With
 *          lse == NULL, bf16 logits, 16-byte aligned rows and 8192 <= V <= 163840 the whole call
 *          is one pass over HBM (the row is held in registers: 4 bytes of traffic per logit);
 *          otherwise a forward pass into the workspace precedes the gradient pass.
 * entropy  f32[T] from aero_logprob_fwd; read only when lse != NULL and entropy_coef != 0
 *          (AERO_ERR_NULL if missing then), may be NULL otherwise.
 * old_logprob f32[T]; token_rollout i32[T] (AERO_ROW_PADDING / AERO_ROW_UNTOUCHED = no rollout); adv, weight f32[R].
 * entropy_coef  c above; 0 switches the term off (NaN: AERO_ERR_SHAPE).
 * kl_coef, ref_logprob  beta above and f32[T] log pi_ref of the sampled tokens; ref_logprob is read
 *          only when kl_coef != 0 (AERO_ERR_NULL if missing then).
 * Outputs  loss f32[1] (deterministic: fixed-order reduction); clip_frac f32[1] or NULL
 *          (clipped tokens / tokens with A != 0 and w != 0); dlogits or NULL (loss only);
 *          logprob_out f32[T] or NULL: current log-prob of the tokens that carry signal, 0 elsewhere;
 *          entropy_out, lse_out f32[T] or NULL: allowed only with lse == NULL (AERO_ERR_NULL
 *          otherwise); when either is given, logprob_out / entropy_out / lse_out are written for
 *          every row with a valid rollout index and sampled token (as aero_logprob_fwd would),
 *          0 elsewhere.
 * workspace: aero_workspace_bytes(AERO_OP_GRPO_LOSS_BWD, T, V, 0, R, 0).
 */
aero_status aero_grpo_loss_bwd(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
    const int32_t* targets, const float* lse /*nullable*/, const float* entropy /*nullable*/,
    const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight, int32_t R,
    float eps_lo, float eps_hi, float grad_scale, float entropy_coef,
    float kl_coef, const float* ref_logprob /*nullable*/,
    float* loss, float* clip_frac /*nullable*/, float* logprob_out /*nullable*/,
    float* entropy_out /*nullable*/, float* lse_out /*nullable*/,
    void* dlogits /*nullable*/, int32_t* err_flag /*nullable*/,
    void* workspace, size_t workspace_bytes, void* stream);

/*
 * aero_grpo_loss_bwd for callers that cannot allocate device memory and so cannot bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and status codes as aero_grpo_loss_bwd, minus `workspace` /
 * `workspace_bytes`: the scratch is a fixed array of device memory inside the library
 * (9 * 4 * AERO_NOALLOC_MAX_T + 256 bytes, about 2.3 MB, held on every GPU the library runs on
 * until the process ends).  The call allocates and frees nothing.
 *   - T > AERO_NOALLOC_MAX_T returns AERO_ERR_LIMIT and enqueues nothing.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on the same GPU
 *     (different streams, different threads) race; order them on one stream.  The array keeps the
 *     previous call's contents; the call clears what it needs cleared itself.
 *   - The first call on a device looks up the array's address on that device (and may load the
 *     code object): make it once outside any graph capture.
 */
#define AERO_NOALLOC_MAX_T 65536
aero_status aero_grpo_loss_bwd_noalloc(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
    const int32_t* targets, const float* lse /*nullable*/, const float* entropy /*nullable*/,
    const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight, int32_t R,
    float eps_lo, float eps_hi, float grad_scale, float entropy_coef,
    float kl_coef, const float* ref_logprob /*nullable*/,
    float* loss, float* clip_frac /*nullable*/, float* logprob_out /*nullable*/,
    float* entropy_out /*nullable*/, float* lse_out /*nullable*/,
    void* dlogits /*nullable*/, int32_t* err_flag /*nullable*/, void* stream);

/*
 * The same statistics, loss and gradients with the LM head fused in: logits are
 * z = hidden @ weight^T (no bias, fp32 accumulation of bf16 products) and are never
 * written to memory as a [T, V] tensor.
 *
 * Defines: App. C (the policy is the softmax of the model's final linear layer: pi = softmax(h W^T),
 * temperature 1, Table 8); Eq. 2 (clipped surrogate over the tokens of the kept rollouts, weights
 * 1/N and 1/|o_i|, optional - beta D_KL term); App. A.1 (grad rho = rho grad log pi, clipped tokens
 * contribute nothing, d log pi(y) / d z_j = 1[j = y] - pi_j), carried one step further through
 * z = h W^T: dhidden = dz W, dweight = dz^T h.
 *
 * hidden   bf16 [T, H] row-major, weight bf16 [V, H] row-major, both 16-byte aligned, H % 8 == 0.
 * Forward outputs  logprob[T], lse[T] f32, entropy[T] f32 or NULL.
 * Backward part (old_logprob .. dweight; pass old_logprob == NULL for forward only):
 *   loss f32[1]; dhidden bf16 [T, H] (16-byte aligned) = dz @ weight; dweight [V, H] = dz^T @ hidden in
 *   dweight_dtype (AERO_F32 or AERO_BF16, optionally | AERO_DW_ACCUMULATE), with dz as defined for aero_grpo_loss_bwd
 *   (entropy_coef and kl_coef / ref_logprob included: the entropy of the forward part is used,
 *   also when the `entropy` output is NULL).
 * Rows whose target or rollout index is negative take no part in the contraction (their outputs, the
 * dhidden row included, are 0; AERO_ROW_UNTOUCHED means the same as AERO_ROW_PADDING here); a
 * target >= V is treated the same way and raises AERO_DERR_BAD_TARGET in err_flag.
 * workspace: aero_workspace_bytes(AERO_OP_LMHEAD_FUSED, T, V, H, R, 0) bytes of device memory,
 * 256-byte aligned, owned by the caller, contents undefined before and after the call.
 * Errors: AERO_ERR_SHAPE (T < 0, V < 1 or > 2^24, H < 8, H % 8 != 0, or a padded backward
 * operand of 4 GiB or more: H, T or the vocabulary chunk too large for 32-bit offsets),
 * AERO_ERR_DTYPE (dweight_dtype), AERO_ERR_NULL, AERO_ERR_ALIGN, AERO_ERR_WORKSPACE,
 * AERO_ERR_HIP (launch failure).  Asynchronous on `stream`; nothing is allocated.
 */
aero_status aero_lmhead_logprob_fused(
    const void* hidden, const void* weight, int64_t T, int32_t H, int32_t V,
    const int32_t* targets,
    float* logprob, float* entropy /*nullable*/, float* lse,
    const float* old_logprob /*nullable => forward only*/, const int32_t* token_rollout,
    const float* adv, const float* weight_rollout, int32_t R,
    float eps_lo, float eps_hi, float grad_scale, float entropy_coef,
    float kl_coef, const float* ref_logprob /*nullable*/,
    float* loss, float* clip_frac /*nullable*/, void* dhidden, void* dweight, int32_t dweight_dtype,
    int32_t* err_flag /*nullable*/,
    void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AERO_H */
