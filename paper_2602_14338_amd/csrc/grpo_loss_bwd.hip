// Clipped-ratio surrogate (Eq. 2, beta = 0, loss = -J) and its gradient w.r.t. the logits
// (App. A.1: grad rho = rho grad log pi; clipped tokens contribute nothing).
//
// Three steps on one stream:
//   token terms  one thread per token: ratio, clip decision, loss term, g_t = dloss/dlogprob
//   loss reduce  one workgroup, fixed summation order (bitwise reproducible), fp64 accumulator
//   dlogits      one workgroup per row: dz = g_t (onehot - exp(z - lse)); rows with g_t == 0
//                are not read, they are only filled with +0 (rows marked AERO_ROW_UNTOUCHED: not even that)
// Entropy bonus (Table 8 lists a coefficient; aggregated here with Eq. 2's weights): with a
// coefficient c != 0 every token of a rollout with w != 0 also contributes -c w H_t to the loss
// and e_t pi_j (ln pi_j + H_t), e_t = grad_scale c w, to its gradient row.  A row is then
// dz_j = pi_j (a z_j + b) + g 1[j = y]  with a = e_t, b = e_t (H_t - lse_t) - g_t, and the
// kernels with ENT = true read (a, b) per row; with c == 0 the ENT = false kernels run.
// KL penalty (Eq. 2's beta term, per-token estimator exp(d) - d - 1 with d = log pi_ref(y) - log pi(y)):
// a per-token scalar like the surrogate, so it only adds to the loss term and to g_t.
#include <mutex>

#include "aero_device.h"

namespace aero {

aero_status logprob_fwd_launch(const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
                               const int32_t* targets, const uint8_t* row_active, float* logprob,
                               float* entropy, float* lse, int32_t* err_flag, hipStream_t s);
bool single_pass_applicable(int32_t dtype, int V, int64_t ld, const void* logits, const void* dlogits);
aero_status single_pass_launch(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                               const float* old_logprob, const int32_t* token_rollout, const float* adv,
                               const float* weight, int R, float eps_lo, float eps_hi, float grad_scale,
                               float ent_coef, float kl_coef, const float* ref_logprob, int stats_all, float* g,
                               float* term, int32_t* flag, float* logprob_out, float* entropy_out, float* lse_out,
                               void* dlogits, int32_t* err_flag, int32_t* row_counter, int32_t* row_order,
                               hipStream_t s);

// ---------------------------------------------------------------- workspace layout
struct LossWorkspace {
  float* g;          // [T] dloss / dlogprob; -0.0 marks a row whose gradient row is not to be written at all
  float* loss_term;  // [T]
  int32_t* flag;     // [T] 0 = no signal, 1 = unclipped, 2 = clipped
  float* lse;        // [T] used when the caller gives none
  float* lp_tmp;     // [T] sink for the forward pass's log-prob when lse is recomputed; the row order (i32) of
                     //     the streaming single-pass kernel, which does not use that sink
  uint8_t* signal;   // [T] rows that carry signal, so the recomputing forward pass skips the rest
  float* ea;         // [T] entropy bonus: a_t = grad_scale c w
  float* eb;         // [T] entropy bonus: b_t = a_t (H_t - lse_t) - g_t
  float* ent;        // [T] entropy of the rows when the caller passes no array for it
  int32_t* counter;  // [4] counters of the streaming single-pass kernel
};
constexpr size_t kAlign = 256;
constexpr size_t seg(int64_t T) { return (size_t(T) * 4 + kAlign - 1) / kAlign * kAlign; }
constexpr size_t loss_workspace_bytes_c(int64_t T) { return 9 * seg(T) + kAlign; }
size_t loss_workspace_bytes(int64_t T) { return loss_workspace_bytes_c(T); }
inline LossWorkspace carve(void* ws, int64_t T) {
  char* p = reinterpret_cast<char*>(ws);
  const size_t s = seg(T);
  return LossWorkspace{reinterpret_cast<float*>(p), reinterpret_cast<float*>(p + s),
                       reinterpret_cast<int32_t*>(p + 2 * s), reinterpret_cast<float*>(p + 3 * s),
                       reinterpret_cast<float*>(p + 4 * s), reinterpret_cast<uint8_t*>(p + 5 * s),
                       reinterpret_cast<float*>(p + 6 * s), reinterpret_cast<float*>(p + 7 * s),
                       reinterpret_cast<float*>(p + 8 * s), reinterpret_cast<int32_t*>(p + 9 * s)};
}

// ---------------------------------------------------------------- which rows carry signal
// stats_all: every valid row (rollout index and sampled token in range) needs statistics;
// every_weighted: rows of rollouts with advantage 0 count too (entropy bonus)
__global__ __launch_bounds__(256) void k_signal_mask(
    int64_t T, int V, const int32_t* __restrict__ targets, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R, int stats_all, int every_weighted,
    uint8_t* __restrict__ signal) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (t >= T) return;
  const int i = token_rollout[t], y = targets[t];
  const bool valid = i >= 0 && i < R && y >= 0 && y < V;
  signal[t] = (valid && (stats_all || (weight[i] != 0.f && (every_weighted || adv[i] != 0.f)))) ? 1 : 0;
}

// ---------------------------------------------------------------- token terms
// LP_GIVEN: the current log-prob is read from `logprob_in` (fused LM-head path) instead of
// being formed as z[t, y] - lse[t].
template <int DT, bool LP_GIVEN>
__global__ __launch_bounds__(256) void k_token_terms(
    const void* __restrict__ logits, int64_t T, int V, int64_t ld, const int32_t* __restrict__ targets,
    const float* __restrict__ lse, const float* __restrict__ logprob_in,
    const float* __restrict__ old_logprob, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R,
    float eps_lo, float eps_hi, float grad_scale, float ent_coef, const float* __restrict__ entropy,
    float kl_coef, const float* __restrict__ ref_logprob,
    float* __restrict__ g_out, float* __restrict__ term_out, int32_t* __restrict__ flag_out,
    float* __restrict__ ea_out, float* __restrict__ eb_out,
    float* __restrict__ logprob_out, int32_t* __restrict__ err_flag) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (t >= T) return;
  const int i = token_rollout[t];
  const int y = targets[t];
  float g = 0.f, term = 0.f, lp = 0.f, ea = 0.f, eb = 0.f;
  int flag = 0;
  if (i < 0 || y < 0) {
    // padding / ignored row: whatever its other index holds is not looked at
  } else if (i >= R || y >= V) {
    if (err_flag) atomicOr(err_flag, i >= R ? AERO_DERR_BAD_ROLLOUT : AERO_DERR_BAD_TARGET);
  } else {
    const float A = adv[i], w = weight[i];
    if (w != 0.f && (A != 0.f || ent_coef != 0.f || kl_coef != 0.f)) {   // decided before the ratio is touched
      if constexpr (LP_GIVEN) {
        lp = logprob_in[t];
      } else {
        lp = load_elt<DT>(logits, int64_t(t) * ld + y) - lse[t];
      }
      if (A != 0.f) {
        const float rho = expf(lp - old_logprob[t]);
        const float lo = 1.f - eps_lo, hi = 1.f + eps_hi;
        const float clipped = fminf(fmaxf(rho, lo), hi);
        const float s = fminf(rho * A, clipped * A);
        const bool unclipped = A > 0.f ? (rho <= hi) : (rho >= lo);
        term = -w * s;
        g = unclipped ? -grad_scale * w * A * rho : 0.f;
        flag = unclipped ? 1 : 2;
      }
      if (kl_coef != 0.f) {   // Eq. 2's beta term, per-token estimator exp(d) - d - 1, d = log pi_ref - log pi
        const float d = ref_logprob[t] - lp;
        const float ed = expf(d);
        term += kl_coef * w * (ed - d - 1.f);
        g += grad_scale * kl_coef * w * (1.f - ed);
      }
      if (ent_coef != 0.f) {
        const float H = entropy[t];
        term -= ent_coef * w * H;
        ea = grad_scale * ent_coef * w;
        eb = ea * (H - lse[t]) - g;
      }
    }
  }
  // the sign of a zero carries "leave the gradient row alone" to the gradient kernels, which have g_t in hand
  // before anything else: +0 = fill the row with zeros, -0 = do not write it
  if (g == 0.f) g = (i == AERO_ROW_UNTOUCHED) ? -0.f : 0.f;
  g_out[t] = g;
  term_out[t] = term;
  flag_out[t] = flag;
  if (ea_out) {
    ea_out[t] = ea;
    eb_out[t] = eb;
  }
  if (logprob_out) logprob_out[t] = lp;
}

// ---------------------------------------------------------------- loss reduce
constexpr int kReduceNT = 1024;
__global__ __launch_bounds__(kReduceNT) void k_loss_reduce(
    const float* __restrict__ term, const int32_t* __restrict__ flag, int64_t T,
    float* __restrict__ loss, float* __restrict__ clip_frac) {
  __shared__ double s_sum[kReduceNT];
  __shared__ int s_sig[kReduceNT], s_clip[kReduceNT];
  double acc = 0.0;
  int nsig = 0, nclip = 0;
  for (int64_t t = threadIdx.x; t < T; t += kReduceNT) {   // fixed order per thread
    acc += double(term[t]);
    const int f = flag[t];
    nsig += f != 0;
    nclip += f == 2;
  }
  s_sum[threadIdx.x] = acc;
  s_sig[threadIdx.x] = nsig;
  s_clip[threadIdx.x] = nclip;
  __syncthreads();
  for (int off = kReduceNT / 2; off > 0; off >>= 1) {      // fixed tree
    if (threadIdx.x < off) {
      s_sum[threadIdx.x] += s_sum[threadIdx.x + off];
      s_sig[threadIdx.x] += s_sig[threadIdx.x + off];
      s_clip[threadIdx.x] += s_clip[threadIdx.x + off];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    loss[0] = float(s_sum[0]);
    if (clip_frac) clip_frac[0] = s_sig[0] ? float(s_clip[0]) / float(s_sig[0]) : 0.f;
  }
}

// ---------------------------------------------------------------- dlogits
// dz_j = s(z_j) * exp(z_j - lse) (+ g at the sampled token), s = -g, or a z_j + b with the entropy term.
template <bool ENT>
__device__ __forceinline__ float grad_elt(float z, float a, float b, float c) {
  return (ENT ? fmaf(a, z, b) : b) * exp2_fast(fmaf(z, kLog2e, c));
}

// One 16-byte vector of logits -> one of gradient; k = index of the vector in its row.
template <int DT, bool ENT>
__device__ __forceinline__ u32x4_t dlogits_vec(const u32x4_t& v, int k, int y, float g, float a, float b, float c) {
  constexpr int E = Storage<DT>::kPerVec;
  float z[E], d[E];
  unpack_vec<DT>(v, z);
#pragma unroll
  for (int e = 0; e < E; ++e) d[e] = grad_elt<ENT>(z[e], a, b, c);
  if (k == y / E) {
#pragma unroll
    for (int e = 0; e < E; ++e) d[e] += (e == y % E) ? g : 0.f;
  }
  return pack_vec<DT>(d);
}

// ENT: the row also carries the entropy-bonus term, dz_j = pi_j (a z_j + b) + g 1[j = y].
template <int NT, int DT, bool VEC, bool ENT>
__global__ __launch_bounds__(NT) void k_dlogits(
    const void* logits, int64_t T, int V, int64_t ld, const int32_t* __restrict__ targets,
    const float* __restrict__ lse, const float* __restrict__ g_arr, const float* __restrict__ ea,
    const float* __restrict__ eb, void* dlogits) {
  const int64_t t = blockIdx.x;
  const float g = g_arr[t];
  float a = 0.f;
  if constexpr (ENT) a = ea[t];
  constexpr size_t kEltBytes = Storage<DT>::kBytes;
  constexpr int E = Storage<DT>::kPerVec;
  const size_t row_off = size_t(t) * size_t(ld) * kEltBytes;
  const char* zrow = reinterpret_cast<const char*>(logits) + row_off;
  char* drow = reinterpret_cast<char*>(dlogits) + row_off;
  const int tid = threadIdx.x;

  if (g == 0.f && a == 0.f) {   // uniform over the workgroup: nothing to read
    if (__float_as_uint(g) >> 31) return;   // -0: the row is not to be written
    if constexpr (VEC) {
      u32x4_t* dv = reinterpret_cast<u32x4_t*>(drow);
      const int nvec = V / E;
      const u32x4_t zero = {0u, 0u, 0u, 0u};
      for (int i = tid; i < nvec; i += NT) __builtin_nontemporal_store(zero, dv + i);
      const int j = nvec * E + tid;
      if (j < V) store_elt<DT>(drow, j, 0.f);
    } else {
      for (int j = tid; j < V; j += NT) store_elt<DT>(drow, j, 0.f);
    }
    return;
  }

  const int y = targets[t];
  const float c = -lse[t] * kLog2e;
  float b = -g;
  if constexpr (ENT) b = eb[t];
  auto grad = [&](float z, int j) -> float {
    const float d = grad_elt<ENT>(z, a, b, c);
    return j == y ? d + g : d;
  };
  if constexpr (VEC) {
    const u32x4_t* zv = reinterpret_cast<const u32x4_t*>(zrow);
    u32x4_t* dv = reinterpret_cast<u32x4_t*>(drow);
    const int nvec = V / E;
    constexpr int UNROLL = 4;
    int i = tid;
    for (; i + (UNROLL - 1) * NT < nvec; i += UNROLL * NT) {
      u32x4_t v[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(zv + i + u * NT);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u)
        __builtin_nontemporal_store(dlogits_vec<DT, ENT>(v[u], i + u * NT, y, g, a, b, c), dv + i + u * NT);
    }
    for (; i < nvec; i += NT) {
      u32x4_t v = __builtin_nontemporal_load(zv + i);
      __builtin_nontemporal_store(dlogits_vec<DT, ENT>(v, i, y, g, a, b, c), dv + i);
    }
    const int j = nvec * E + tid;
    if (j < V) store_elt<DT>(drow, j, grad(load_elt<DT>(zrow, j), j));
  } else {
    for (int j = tid; j < V; j += NT) store_elt<DT>(drow, j, grad(load_elt<DT>(zrow, j), j));
  }
}

// Long aligned rows: one 16-byte vector per thread, (row, segment) per workgroup.  Workgroups
// are small and start in address order, so the whole GPU sweeps the tensor as one linear stream
// of reads and one of writes (a workgroup that loops over its row reaches 5.2 TB/s, this form
// 5.7; two or four vectors per thread were 8 % slower, 512 and 1024 threads 1-2 % slower).  The
// vector load is issued as soon as g_t is known, ahead of the other per-row scalars: with
// one load per thread every dependent scalar fetch in front of it costs throughput (7 % here).
constexpr int kSegNT = 256;
constexpr int kSegVPT = 1;
constexpr int kSegVecs = kSegNT * kSegVPT;   // vectors per segment

template <int DT, bool ENT>
__global__ __launch_bounds__(kSegNT) void k_dlogits_seg(
    const void* logits, int V, int64_t ld, int segs, const int32_t* __restrict__ targets,
    const float* __restrict__ lse, const float* __restrict__ g_arr, const float* __restrict__ ea,
    const float* __restrict__ eb, void* dlogits) {
  constexpr int E = Storage<DT>::kPerVec;
  constexpr size_t kEltBytes = Storage<DT>::kBytes;
  const int64_t t = blockIdx.x / segs;
  const int seg = blockIdx.x % segs;
  const float g = g_arr[t];
  float a = 0.f;
  if constexpr (ENT) a = ea[t];
  const size_t row_off = size_t(t) * size_t(ld) * kEltBytes;
  const char* zrow = reinterpret_cast<const char*>(logits) + row_off;
  char* drow = reinterpret_cast<char*>(dlogits) + row_off;
  const int nvec = V / E;
  const int k0 = seg * kSegVecs + threadIdx.x;
  const int j = nvec * E + threadIdx.x;          // ragged tail, done by segment 0
  const bool tail = seg == 0 && j < V;
  if (g == 0.f && a == 0.f) {   // uniform over the workgroup: nothing to read
    if (__float_as_uint(g) >> 31) return;   // -0: the row is not to be written
#pragma unroll
    for (int i = 0; i < kSegVPT; ++i)
      if (k0 + i * kSegNT < nvec) reinterpret_cast<u32x4_t*>(drow)[k0 + i * kSegNT] = u32x4_t{0u, 0u, 0u, 0u};
    if (tail) store_elt<DT>(drow, j, 0.f);
    return;
  }
  u32x4_t v[kSegVPT];
#pragma unroll
  for (int i = 0; i < kSegVPT; ++i)
    if (k0 + i * kSegNT < nvec) v[i] = reinterpret_cast<const u32x4_t*>(zrow)[k0 + i * kSegNT];
  const int y = targets[t];
  const float c = -lse[t] * kLog2e;
  float b = -g;
  if constexpr (ENT) b = eb[t];
#pragma unroll
  for (int i = 0; i < kSegVPT; ++i) {
    const int k = k0 + i * kSegNT;
    if (k < nvec) reinterpret_cast<u32x4_t*>(drow)[k] = dlogits_vec<DT, ENT>(v[i], k, y, g, a, b, c);
  }
  if (tail) {
    float d = grad_elt<ENT>(load_elt<DT>(zrow, j), a, b, c);
    if (j == y) d += g;
    store_elt<DT>(drow, j, d);
  }
}

template <int DT, bool VEC, bool ENT>
static void dispatch_dlogits(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                             const float* lse, const float* g, const float* ea, const float* eb, void* dlogits,
                             hipStream_t s) {
  const int per_vec = VEC ? Storage<DT>::kPerVec : 1;
  const int64_t work = (V + per_vec - 1) / per_vec;
  if constexpr (VEC) {
    const int64_t segs = (V / per_vec + kSegVecs - 1) / kSegVecs;
    if (work > 16 * 256 && T * segs < (int64_t(1) << 31)) {
      hipLaunchKernelGGL((k_dlogits_seg<DT, ENT>), dim3(unsigned(T * segs)), dim3(kSegNT), 0, s, logits, V, ld,
                         int(segs), targets, lse, g, ea, eb, dlogits);
      return;
    }
  }
  if (work <= 4 * 64)
    hipLaunchKernelGGL((k_dlogits<64, DT, VEC, ENT>), dim3((unsigned)T), dim3(64), 0, s, logits, T, V, ld, targets,
                       lse, g, ea, eb, dlogits);
  else if (work <= 16 * 256)
    hipLaunchKernelGGL((k_dlogits<256, DT, VEC, ENT>), dim3((unsigned)T), dim3(256), 0, s, logits, T, V, ld, targets,
                       lse, g, ea, eb, dlogits);
  else
    hipLaunchKernelGGL((k_dlogits<512, DT, VEC, ENT>), dim3((unsigned)T), dim3(512), 0, s, logits, T, V, ld, targets,
                       lse, g, ea, eb, dlogits);
}

template <bool ENT>
static void dispatch_dlogits_dtype(int32_t dtype, bool vec, const void* logits, int64_t T, int V, int64_t ld,
                                   const int32_t* targets, const float* lse, const float* g, const float* ea,
                                   const float* eb, void* dlogits, hipStream_t s) {
  if (dtype == AERO_BF16) {
    if (vec) dispatch_dlogits<kBF16, true, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
    else dispatch_dlogits<kBF16, false, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
  } else if (dtype == AERO_F16) {
    if (vec) dispatch_dlogits<kF16, true, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
    else dispatch_dlogits<kF16, false, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
  } else if (dtype == AERO_F8E4M3) {
    if (vec) dispatch_dlogits<kF8, true, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
    else dispatch_dlogits<kF8, false, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
  } else {
    if (vec) dispatch_dlogits<kF32, true, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
    else dispatch_dlogits<kF32, false, ENT>(logits, T, V, ld, targets, lse, g, ea, eb, dlogits, s);
  }
}

// Shared with the fused LM-head path: token terms from given log-probs, then the reduction.
aero_status token_terms_from_logprob(int64_t T, int V, const int32_t* targets, const float* logprob,
                                     const float* lse, const float* entropy, const float* old_logprob,
                                     const int32_t* token_rollout, const float* adv, const float* weight, int R,
                                     float eps_lo, float eps_hi, float grad_scale, float ent_coef, float kl_coef,
                                     const float* ref_logprob, float* g, float* term, int32_t* flag, float* ea,
                                     float* eb, float* loss, float* clip_frac, int32_t* err_flag, hipStream_t s) {
  const unsigned blocks = unsigned((T + 255) / 256);
  if (T > 0)
    hipLaunchKernelGGL((k_token_terms<kBF16, true>), dim3(blocks), dim3(256), 0, s, nullptr, T, V, int64_t(0),
                       targets, lse, logprob, old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi,
                       grad_scale, ent_coef, entropy, kl_coef, ref_logprob, g, term, flag, ea, eb, nullptr, err_flag);
  hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(kReduceNT), 0, s, term, flag, T, loss, clip_frac);
  return launch_status();
}

// The loss call proper; both entry points below end here.
static aero_status loss_bwd_run(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld, const int32_t* targets,
    const float* lse, const float* entropy, const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight, int32_t R, float eps_lo, float eps_hi, float grad_scale,
    float entropy_coef, float kl_coef, const float* ref_logprob, float* loss, float* clip_frac, float* logprob_out,
    float* entropy_out, float* lse_out, void* dlogits, int32_t* err_flag, void* workspace, size_t workspace_bytes,
    void* stream) {
  const bool ent = entropy_coef != 0.f;
  if (!(entropy_coef == entropy_coef) || !(kl_coef == kl_coef)) return AERO_ERR_SHAPE;   // NaN coefficient
  if (kl_coef != 0.f && T > 0 && !ref_logprob) return AERO_ERR_NULL;
  if (lse && ent && !entropy) return AERO_ERR_NULL;             // H_t must come with the given lse
  if (T < 0 || V < 1 || V > (1 << 24) || ld < V || R < 0 || T > 0x7fffffffLL) return AERO_ERR_SHAPE;
  if (!storage_dtype_ok(dtype)) return AERO_ERR_DTYPE;
  if (!loss) return AERO_ERR_NULL;
  hipStream_t s = as_stream(stream);
  if (T > 0 && (!logits || !targets || !old_logprob || !token_rollout || !adv || !weight)) return AERO_ERR_NULL;
  if (T > 0 && (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0 ||
                workspace_bytes < loss_workspace_bytes(T)))
    return AERO_ERR_WORKSPACE;
  LossWorkspace ws = carve(workspace, T);
  if (T == 0) {
    hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(kReduceNT), 0, s, nullptr, nullptr, T, loss, clip_frac);
    return launch_status();
  }
  const unsigned blocks = unsigned((T + 255) / 256);
  float* lp_dst = logprob_out;   // where the token-terms step may write the signal rows' log-probs
  if (!lse) {
    // statistics are computed here; with entropy_out / lse_out they cover every valid row
    const int stats_all = (entropy_out || lse_out) ? 1 : 0;
    if (single_pass_applicable(dtype, V, ld, logits, dlogits)) {
      const aero_status sp = single_pass_launch(logits, T, V, ld, targets, old_logprob, token_rollout, adv, weight, R,
                                                eps_lo, eps_hi, grad_scale, entropy_coef, kl_coef, ref_logprob, stats_all, ws.g,
                                                ws.loss_term,
                                                ws.flag,
                                                logprob_out, entropy_out, lse_out, dlogits, err_flag, ws.counter,
                                                reinterpret_cast<int32_t*>(ws.lp_tmp), s);
      if (sp != AERO_OK) return sp;
      hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(kReduceNT), 0, s, ws.loss_term, ws.flag, T, loss, clip_frac);
      return launch_status();
    }
    hipLaunchKernelGGL(k_signal_mask, dim3(blocks), dim3(256), 0, s, T, V, targets, token_rollout, adv, weight,
                       R, stats_all, (ent || kl_coef != 0.f) ? 1 : 0, ws.signal);
    float* lse_dst = lse_out ? lse_out : ws.lse;
    float* ent_dst = entropy_out ? entropy_out : (ent ? ws.ent : nullptr);
    aero_status st = logprob_fwd_launch(logits, dtype, T, V, ld, targets, ws.signal,
                                        stats_all && logprob_out ? logprob_out : ws.lp_tmp, ent_dst, lse_dst,
                                        nullptr, s);
    if (st != AERO_OK) return st;
    lse = lse_dst;
    entropy = ent_dst;
    if (stats_all) lp_dst = nullptr;   // already written for every valid row by the forward pass
  } else if (entropy_out || lse_out) {
    return AERO_ERR_NULL;   // these outputs exist only when the statistics are computed here
  }
  auto token_terms = dtype == AERO_BF16 ? k_token_terms<kBF16, false>
                     : dtype == AERO_F16 ? k_token_terms<kF16, false>
                     : dtype == AERO_F8E4M3 ? k_token_terms<kF8, false> : k_token_terms<kF32, false>;
  hipLaunchKernelGGL(token_terms, dim3(blocks), dim3(256), 0, s, logits, T, V, ld, targets, lse,
                     static_cast<const float*>(nullptr), old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi,
                     grad_scale, entropy_coef, entropy, kl_coef, ref_logprob, ws.g, ws.loss_term, ws.flag,
                     ent ? ws.ea : nullptr, ent ? ws.eb : nullptr, lp_dst, err_flag);
  hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(kReduceNT), 0, s, ws.loss_term, ws.flag, T, loss, clip_frac);
  if (dlogits) {
    const size_t elt = storage_bytes(dtype);
    const bool vec = reinterpret_cast<uintptr_t>(logits) % 16 == 0 && reinterpret_cast<uintptr_t>(dlogits) % 16 == 0 &&
                     (size_t(ld) * elt) % 16 == 0;
    if (ent) dispatch_dlogits_dtype<true>(dtype, vec, logits, T, V, ld, targets, lse, ws.g, ws.ea, ws.eb, dlogits, s);
    else dispatch_dlogits_dtype<false>(dtype, vec, logits, T, V, ld, targets, lse, ws.g, nullptr, nullptr, dlogits, s);
  }
  return launch_status();
}

// ---------------------------------------------------------------- library-owned scratch
// For callers that cannot allocate: the workspace of a loss call of up to kStaticMaxT token rows
// lives in device memory that belongs to the loaded code object.  Every GPU holds its own copy of
// the array at its own address, so the address is looked up once per device, with that device
// current, and only that pointer is ever handed to a kernel or a copy.
constexpr int64_t kStaticMaxT = AERO_NOALLOC_MAX_T;
constexpr size_t kStaticScratchBytes = loss_workspace_bytes_c(kStaticMaxT);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static aero_status static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AERO_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return AERO_ERR_HIP;
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return AERO_OK;
}

}  // namespace aero

extern "C" aero_status aero_grpo_loss_bwd(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld, const int32_t* targets,
    const float* lse, const float* entropy, const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight, int32_t R, float eps_lo, float eps_hi, float grad_scale,
    float entropy_coef, float kl_coef, const float* ref_logprob, float* loss, float* clip_frac, float* logprob_out,
    float* entropy_out, float* lse_out, void* dlogits, int32_t* err_flag, void* workspace, size_t workspace_bytes,
    void* stream) {
  return aero::loss_bwd_run(logits, dtype, T, V, ld, targets, lse, entropy, old_logprob, token_rollout, adv, weight, R,
                            eps_lo, eps_hi, grad_scale, entropy_coef, kl_coef, ref_logprob, loss, clip_frac,
                            logprob_out, entropy_out, lse_out, dlogits, err_flag, workspace, workspace_bytes, stream);
}

extern "C" aero_status aero_grpo_loss_bwd_noalloc(
    const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld, const int32_t* targets,
    const float* lse, const float* entropy, const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight, int32_t R, float eps_lo, float eps_hi, float grad_scale,
    float entropy_coef, float kl_coef, const float* ref_logprob, float* loss, float* clip_frac, float* logprob_out,
    float* entropy_out, float* lse_out, void* dlogits, int32_t* err_flag, void* stream) {
  if (T > aero::kStaticMaxT) return AERO_ERR_LIMIT;
  void* ws = nullptr;
  const aero_status st = aero::static_scratch(&ws);
  if (st != AERO_OK) return st;
  return aero::loss_bwd_run(logits, dtype, T, V, ld, targets, lse, entropy, old_logprob, token_rollout, adv, weight, R,
                            eps_lo, eps_hi, grad_scale, entropy_coef, kl_coef, ref_logprob, loss, clip_frac,
                            logprob_out, entropy_out, lse_out, dlogits, err_flag, ws, aero::kStaticScratchBytes, stream);
}
