// Softmax policy statistics per token row: log-partition, log-prob of the sampled token and
// entropy (App. C, softmax policy; the update consumes log pi of the sampled token).
//
// One workgroup owns one row.  The row is streamed once from HBM with 128-bit loads; each
// thread keeps a running (offset, sum exp, sum exp*z) in registers, waves combine with
// cross-lane shuffles and LDS is touched only for the final cross-wave merge.
#include "aero_device.h"

namespace aero {

// Elements per 16-byte vector
template <bool BF16> struct Elt { static constexpr int kPerVec = BF16 ? 8 : 4; };

template <bool BF16>
__device__ __forceinline__ float load_elt(const void* row, int64_t j) {
  if constexpr (BF16) return bf16_to_f32(reinterpret_cast<const uint16_t*>(row)[j]);
  else return reinterpret_cast<const float*>(row)[j];
}

template <bool BF16>
__device__ __forceinline__ void vec_update(RowStat& st, const u32x4_t& v) {
  if constexpr (BF16) {
    float z[8];
    unpack8(v, z);
    stat_update<8>(st, z);
  } else {
    float z[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
    stat_update<4>(st, z);
  }
}

// Streams one row and returns this thread's partial state.  VEC: row base and stride are
// 16-byte aligned.  UNROLL independent 16-byte loads are issued before any is consumed.
template <int NT, bool BF16, bool VEC, int UNROLL>
__device__ __forceinline__ RowStat row_partial(const void* row, int V) {
  RowStat st = stat_identity();
  const int tid = threadIdx.x;
  if constexpr (VEC) {
    constexpr int E = Elt<BF16>::kPerVec;
    const u32x4_t* rv = reinterpret_cast<const u32x4_t*>(row);
    const int nvec = V / E;
    int i = tid;
    for (; i + (UNROLL - 1) * NT < nvec; i += UNROLL * NT) {
      u32x4_t v[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(rv + i + u * NT);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) vec_update<BF16>(st, v[u]);
    }
    for (; i < nvec; i += NT) {
      u32x4_t v = __builtin_nontemporal_load(rv + i);
      vec_update<BF16>(st, v);
    }
    const int j = nvec * E + tid;   // ragged tail shorter than one vector
    if (j < V) {
      float z[1] = {load_elt<BF16>(row, j)};
      stat_update<1>(st, z);
    }
  } else {
    for (int j = tid; j < V; j += NT) {
      float z[1] = {load_elt<BF16>(row, j)};
      stat_update<1>(st, z);
    }
  }
  return st;
}

template <int NT, bool BF16, bool VEC>
__global__ __launch_bounds__(NT) void k_logprob_fwd(
    const void* __restrict__ logits, int64_t T, int V, int64_t ld,
    const int32_t* __restrict__ targets, const uint8_t* __restrict__ row_active,
    float* __restrict__ logprob, float* __restrict__ entropy, float* __restrict__ lse_out,
    int32_t* __restrict__ err_flag) {
  __shared__ RowStat lds[NT / kWave];
  const int64_t t = blockIdx.x;
  const int y = targets[t];
  const bool active = (row_active == nullptr || row_active[t] != 0) && y >= 0 && y < V;
  if (!active) {   // uniform over the workgroup
    if (threadIdx.x == 0) {
      logprob[t] = 0.f;
      lse_out[t] = 0.f;
      if (entropy) entropy[t] = 0.f;
      // a row the caller switched off is ignored whatever its target holds
      if (y >= V && (row_active == nullptr || row_active[t] != 0) && err_flag) atomicOr(err_flag, AERO_DERR_BAD_TARGET);
    }
    return;
  }
  constexpr size_t kEltBytes = BF16 ? 2 : 4;
  const char* row = reinterpret_cast<const char*>(logits) + size_t(t) * size_t(ld) * kEltBytes;
  RowStat st = row_partial<NT, BF16, VEC, 4>(row, V);
  st = stat_block_reduce<NT>(st, lds);
  if (threadIdx.x == 0) {
    const float lse = st.m + logf(st.s);
    const float zy = load_elt<BF16>(row, y);
    logprob[t] = zy - lse;
    lse_out[t] = lse;
    if (entropy) entropy[t] = lse - st.sz / st.s;
  }
}

template <int NT, bool BF16, bool VEC>
static void launch_fwd(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                       const uint8_t* row_active, float* logprob, float* entropy, float* lse,
                       int32_t* err_flag, hipStream_t s) {
  hipLaunchKernelGGL((k_logprob_fwd<NT, BF16, VEC>), dim3((unsigned)T), dim3(NT), 0, s, logits, T, V, ld,
                     targets, row_active, logprob, entropy, lse, err_flag);
}

template <bool BF16, bool VEC>
static void dispatch_nt(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                        const uint8_t* row_active, float* logprob, float* entropy, float* lse,
                        int32_t* err_flag, hipStream_t s) {
  // threads per row: one wave for short rows, more as the row grows
  const int per_vec = VEC ? Elt<BF16>::kPerVec : 1;
  const int64_t work = (V + per_vec - 1) / per_vec;
  if (work <= 4 * 64) launch_fwd<64, BF16, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  else if (work <= 16 * 256) launch_fwd<256, BF16, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  else launch_fwd<512, BF16, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
}

// Internal entry used by the loss call when the caller gives no lse.
aero_status logprob_fwd_launch(const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
                               const int32_t* targets, const uint8_t* row_active, float* logprob,
                               float* entropy, float* lse, int32_t* err_flag, hipStream_t s) {
  if (T == 0) return AERO_OK;
  const size_t elt = dtype == AERO_BF16 ? 2 : 4;
  const bool vec = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((size_t(ld) * elt) % 16 == 0);
  if (dtype == AERO_BF16) {
    if (vec) dispatch_nt<true, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<true, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  } else {
    if (vec) dispatch_nt<false, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<false, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  }
  return launch_status();
}

}  // namespace aero

extern "C" aero_status aero_logprob_fwd(const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
                                        const int32_t* targets, const uint8_t* row_active,
                                        float* logprob, float* entropy, float* lse,
                                        int32_t* err_flag, void* stream) {
  if (T < 0 || V < 1 || V > (1 << 24) || ld < V || T > 0x7fffffffLL) return AERO_ERR_SHAPE;
  if (dtype != AERO_BF16 && dtype != AERO_F32) return AERO_ERR_DTYPE;
  if (T == 0) return AERO_OK;
  if (!logits || !targets || !logprob || !lse) return AERO_ERR_NULL;
  return aero::logprob_fwd_launch(logits, dtype, T, V, ld, targets, row_active, logprob, entropy, lse,
                                  err_flag, aero::as_stream(stream));
}
