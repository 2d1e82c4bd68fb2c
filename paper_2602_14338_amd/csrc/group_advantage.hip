// Group statistics, curated subset, group-relative advantages and loss weights
// (Eq. 1; Sec. 3.2; Sec. 4.1 / Alg. 1 strata; Sec. 4.2 Strategies 2 and 3; App. C categories).
//
// Groups are ragged (CSR offsets).  One wave64 owns one group and walks it in strides of 64,
// so any group size works; counts are integers, the few floating-point statistics are formed
// in fp64 from those counts and rounded once to fp32.  Three launches on one stream:
//   k_group     per group: c, category, keep mask, advantages, weights, kept count
//   k_scan      one workgroup: exclusive scan of the kept counts -> kept_offsets
//   k_compact   per group: kept rollout indices, ascending, written at kept_offsets[q]
// or, for a micro-batch's handful of groups (at most two per wave of one workgroup), the same three
// stages in one launch (k_group_small): the call is latency bound there, and two launches less are
// half of its time.  With more groups the three-launch form wins again (64 groups: 13.5 us against 18.7).
#include "aero_device.h"

namespace aero {

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}
__device__ __forceinline__ float wave_max_f(float v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ float wave_min_f(float v) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, kWave));
  return v;
}

// (key, index) ordering used for down-sampling: smaller key first, ties to the lower index
__device__ __forceinline__ bool before(uint32_t ka, int ia, uint32_t kb, int ib) {
  return ka < kb || (ka == kb && ia < ib);
}

constexpr int kGroupsPerBlock = 4;   // 4 waves of 64

// One group, one wave: everything but the position of its kept rollouts in kept_index.  Returns the
// number of kept rollouts (the same value in every lane).
__device__ __forceinline__ int group_body(
    int q, int lane, const float* __restrict__ rewards, const int32_t* __restrict__ lengths,
    const int32_t* __restrict__ group_offsets, const uint32_t* __restrict__ keys, int Q, int R,
    const aero_adv_params& p, float* __restrict__ adv, float* __restrict__ weight, uint8_t* __restrict__ keep_mask,
    uint8_t* __restrict__ zero_var, uint8_t* __restrict__ category, int32_t* __restrict__ err_flag) {
  int b = group_offsets[q], e = group_offsets[q + 1];
  b = max(0, min(b, R));   // offsets outside [0, R] cannot make the kernel read out of bounds
  e = max(b, min(e, R));
  const int n = e - b;
  const bool curation = p.reject_enable || p.posterior_mode;

  // 1. c = number of rollouts with reward exactly 1
  int c_l = 0, bad_l = 0;
  for (int i = b + lane; i < e; i += kWave) {
    const float r = rewards[i];
    c_l += r == 1.f;
    bad_l += (r != 0.f && r != 1.f);
  }
  const int c = wave_sum_i(c_l);
  if (curation && wave_sum_i(bad_l) && lane == 0 && err_flag) atomicOr(err_flag, AERO_DERR_NONBINARY_REWARD);

  // 2. category by u = c/n against tau, integer compares
  int cat;
  if (c == 0) cat = AERO_CAT_ZERO;
  else if (c == n) cat = AERO_CAT_PERFECT;
  else if (int64_t(c) * p.tau_den < int64_t(n) * p.tau_num) cat = AERO_CAT_PARTIAL;
  else cat = AERO_CAT_GOOD;

  // 3. kept subset.  mode 0: all, 1: none, 2: all correct + m lowest-ranked incorrect,
  //    3: the m lowest-ranked of the whole group
  int mode = 0, m = 0;
  if (p.reject_enable) {
    if (cat == AERO_CAT_PARTIAL) {
      mode = 2;
      m = int(min(int64_t(p.k_ratio) * c, int64_t(n - c)));
    } else if (cat != AERO_CAT_GOOD) {
      mode = p.posterior_mode ? 3 : 1;
      m = min(p.zero_keep, n);
    }
  }
  int nk_l = 0;                    // kept
  double sum_l = 0.0;              // sum of kept rewards
  float mx_l = -INFINITY, mn_l = INFINITY;
  for (int i = b + lane; i < e; i += kWave) {
    const float r = rewards[i];
    bool k;
    if (mode == 0) k = true;
    else if (mode == 1) k = false;
    else if (mode == 2 && r == 1.f) k = true;
    else {
      // rank among the candidates (incorrect rollouts in mode 2, everyone in mode 3)
      const uint32_t ki = keys ? keys[i] : 0u;
      int ahead = 0;
      for (int j = b; j < e && ahead < m; ++j) {
        const bool cand = mode == 3 || rewards[j] != 1.f;
        ahead += cand && before(keys ? keys[j] : 0u, j, ki, i);
      }
      k = ahead < m;
    }
    keep_mask[i] = k ? 1 : 0;
    if (k) {
      ++nk_l;
      sum_l += double(r);
      mx_l = fmaxf(mx_l, r);
      mn_l = fminf(mn_l, r);
    }
  }
  const int nk = wave_sum_i(nk_l);
  const float mx = wave_max_f(mx_l), mn = wave_min_f(mn_l);
  const bool zv = nk == 0 || mx == mn;

  // 4./5. advantages over the kept subset
  double mu = 0.0, inv_sigma = 0.0;
  if (!zv) {
    mu = wave_sum_d(sum_l) / double(nk);
    double ss_l = 0.0;
    for (int i = b + lane; i < e; i += kWave)
      if (keep_mask[i]) {   // written by this same lane above
        const double d = double(rewards[i]) - mu;
        ss_l += d * d;
      }
    inv_sigma = 1.0 / sqrt(wave_sum_d(ss_l) / double(nk));
  } else if (p.posterior_mode && nk > 0) {
    // posterior mean from the observed c, n of the whole group
    mu = (double(c) + double(p.alpha0)) / (double(n) + double(p.alpha0) + double(p.beta0));
    inv_sigma = 1.0 / sqrt(mu * (1.0 - mu));
  }
  const bool signal = !zv || (p.posterior_mode && nk > 0);

  // 6. weights 1 / (Q n' L_i)
  for (int i = b + lane; i < e; i += kWave) {
    const bool k = keep_mask[i] != 0;
    float a = 0.f, w = 0.f;
    if (k) {
      if (signal) a = float((double(rewards[i]) - mu) * inv_sigma);
      const int L = lengths[i];
      if (L > 0) w = float(1.0 / (double(Q) * double(nk) * double(L)));
    }
    adv[i] = a;
    weight[i] = w;
  }
  if (lane == 0) {
    zero_var[q] = zv ? 1 : 0;
    category[q] = uint8_t(cat | (c <= p.s_rescue ? AERO_CAT_RESCUE_BIT : 0));
  }
  return nk;
}

// Kept rollout indices of one group, ascending, written from position `out` on (one wave).
__device__ __forceinline__ void compact_body(int q, int lane, const int32_t* __restrict__ group_offsets,
                                             const uint8_t* __restrict__ keep_mask, int out, int R,
                                             int32_t* __restrict__ kept_index) {
  int b = group_offsets[q], e = group_offsets[q + 1];
  b = max(0, min(b, R));
  e = max(b, min(e, R));
  for (int base = b; base < e; base += kWave) {   // trip count is uniform over the wave
    const int i = base + lane;
    const bool k = i < e && keep_mask[i] != 0;
    const uint64_t bal = __ballot(k);
    if (k) kept_index[out + __popcll(bal & ((uint64_t(1) << lane) - 1))] = i;
    out += __popcll(bal);
  }
}

__global__ __launch_bounds__(kGroupsPerBlock* kWave) void k_group(
    const float* __restrict__ rewards, const int32_t* __restrict__ lengths,
    const int32_t* __restrict__ group_offsets, const uint32_t* __restrict__ keys, int Q, int R,
    aero_adv_params p, float* __restrict__ adv, float* __restrict__ weight, uint8_t* __restrict__ keep_mask,
    int32_t* __restrict__ kept_offsets, uint8_t* __restrict__ zero_var, uint8_t* __restrict__ category,
    int32_t* __restrict__ err_flag) {
  const int lane = threadIdx.x % kWave;
  const int q = blockIdx.x * kGroupsPerBlock + threadIdx.x / kWave;
  if (q >= Q) return;   // whole wave leaves together
  const int nk = group_body(q, lane, rewards, lengths, group_offsets, keys, Q, R, p, adv, weight, keep_mask, zero_var,
                            category, err_flag);
  if (lane == 0) kept_offsets[q + 1] = nk;
}

// Exclusive scan of counts held in kept_offsets[1..Q] (in place), kept_offsets[0] = 0.
constexpr int kScanNT = 1024;
__global__ __launch_bounds__(kScanNT) void k_scan(int32_t* kept_offsets, int Q) {
  __shared__ int part[kScanNT];
  const int per = (Q + kScanNT - 1) / kScanNT;
  const int lo = min(Q, int(threadIdx.x) * per), hi = min(Q, lo + per);
  int s = 0;
  for (int q = lo; q < hi; ++q) s += kept_offsets[q + 1];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int off = 1; off < kScanNT; off <<= 1) {   // inclusive Hillis-Steele over thread sums
    int v = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
    __syncthreads();
    part[threadIdx.x] += v;
    __syncthreads();
  }
  int run = threadIdx.x ? part[threadIdx.x - 1] : 0;
  for (int q = lo; q < hi; ++q) {
    run += kept_offsets[q + 1];
    kept_offsets[q + 1] = run;
  }
  if (threadIdx.x == 0) kept_offsets[0] = 0;
}

__global__ __launch_bounds__(kGroupsPerBlock* kWave) void k_compact(
    const int32_t* __restrict__ group_offsets, const uint8_t* __restrict__ keep_mask,
    const int32_t* __restrict__ kept_offsets, int Q, int R, int32_t* __restrict__ kept_index) {
  const int lane = threadIdx.x % kWave;
  const int q = blockIdx.x * kGroupsPerBlock + threadIdx.x / kWave;
  if (q >= Q) return;
  compact_body(q, lane, group_offsets, keep_mask, kept_offsets[q], R, kept_index);
}

// The three stages in one workgroup of 16 waves, for Q <= kSmallQ groups: wave w takes groups w and w + 16;
// the kept counts and their scan stay in LDS; every wave then places the kept indices of the groups it
// processed (it reads back the keep mask its own lanes wrote).
constexpr int kSmallQ = 32, kSmallR = 1 << 16, kSmallNT = 1024;
__global__ __launch_bounds__(kSmallNT) void k_group_small(
    const float* __restrict__ rewards, const int32_t* __restrict__ lengths,
    const int32_t* __restrict__ group_offsets, const uint32_t* __restrict__ keys, int Q, int R,
    aero_adv_params p, float* __restrict__ adv, float* __restrict__ weight, uint8_t* __restrict__ keep_mask,
    int32_t* __restrict__ kept_index, int32_t* __restrict__ kept_offsets, uint8_t* __restrict__ zero_var,
    uint8_t* __restrict__ category, int32_t* __restrict__ err_flag) {
  __shared__ int start[kSmallQ + 1];   // counts, then exclusive offsets
  __shared__ int part[kSmallNT / kWave];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  constexpr int kWaves = kSmallNT / kWave;
  for (int q = wave; q < Q; q += kWaves) {
    const int nk = group_body(q, lane, rewards, lengths, group_offsets, keys, Q, R, p, adv, weight, keep_mask, zero_var,
                              category, err_flag);
    if (lane == 0) start[q] = nk;
  }
  __syncthreads();
  // exclusive scan of start[0 .. Q): two entries per thread, shuffles inside a wave, the 16 wave totals through LDS
  const int q0 = 2 * tid, q1 = 2 * tid + 1;
  const int c0 = q0 < Q ? start[q0] : 0, c1 = q1 < Q ? start[q1] : 0;
  int incl = c0 + c1;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int v = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += v;
  }
  if (lane == kWave - 1) part[wave] = incl;
  __syncthreads();   // also: every read of start[] above precedes the writes below
  int before_me = incl - (c0 + c1), total = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    before_me += w < wave ? part[w] : 0;
    total += part[w];
  }
  if (q0 < Q) start[q0] = before_me;
  if (q1 < Q) start[q1] = before_me + c0;
  if (tid == 0) start[Q] = total;
  __syncthreads();
  for (int q = tid; q <= Q; q += kSmallNT) kept_offsets[q] = start[q];
  for (int q = wave; q < Q; q += kWaves) compact_body(q, lane, group_offsets, keep_mask, start[q], R, kept_index);
}

}  // namespace aero

extern "C" aero_status aero_group_advantage(
    const float* rewards, const int32_t* lengths, const int32_t* group_offsets,
    const uint32_t* keep_priority, int32_t Q, int32_t R, const aero_adv_params* p, float* adv,
    float* weight, uint8_t* keep_mask, int32_t* kept_index, int32_t* kept_offsets,
    uint8_t* group_zero_var, uint8_t* group_category, int32_t* err_flag, void* stream) {
  using namespace aero;
  if (Q < 0 || R < 0) return AERO_ERR_SHAPE;
  if (!p || !group_offsets || !kept_offsets) return AERO_ERR_NULL;
  if (p->k_ratio < 1 || p->tau_den < 1 || p->tau_num < 0 || p->zero_keep < 0 || p->s_rescue < 0) return AERO_ERR_SHAPE;
  if (Q > 0 && (!group_zero_var || !group_category)) return AERO_ERR_NULL;
  if (R > 0 && (!rewards || !lengths || !adv || !weight || !keep_mask || !kept_index)) return AERO_ERR_NULL;
  hipStream_t s = as_stream(stream);
  if (Q > 0 && Q <= kSmallQ && R <= kSmallR) {
    hipLaunchKernelGGL(k_group_small, dim3(1), dim3(kSmallNT), 0, s, rewards, lengths, group_offsets, keep_priority, Q, R,
                       *p, adv, weight, keep_mask, kept_index, kept_offsets, group_zero_var, group_category, err_flag);
    return launch_status();
  }
  const unsigned blocks = unsigned((Q + kGroupsPerBlock - 1) / kGroupsPerBlock);
  if (Q > 0)
    hipLaunchKernelGGL(k_group, dim3(blocks), dim3(kGroupsPerBlock * kWave), 0, s, rewards, lengths, group_offsets,
                       keep_priority, Q, R, *p, adv, weight, keep_mask, kept_offsets, group_zero_var,
                       group_category, err_flag);
  hipLaunchKernelGGL(k_scan, dim3(1), dim3(kScanNT), 0, s, kept_offsets, Q);
  if (Q > 0)
    hipLaunchKernelGGL(k_compact, dim3(blocks), dim3(kGroupsPerBlock * kWave), 0, s, group_offsets, keep_mask,
                       kept_offsets, Q, R, kept_index);
  return launch_status();
}
