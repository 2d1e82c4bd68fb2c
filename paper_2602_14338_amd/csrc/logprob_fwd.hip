// Softmax policy statistics per token row: log-partition, log-prob of the sampled token and
// entropy (App. C, softmax policy; the update consumes log pi of the sampled token).
//
// One workgroup owns one row.  The row is streamed once from HBM with 128-bit loads; each
// thread keeps a running (offset, sum exp, sum exp*z) in registers, waves combine with
// cross-lane shuffles and LDS is touched only for the final cross-wave merge.
#include "aero_device.h"

namespace aero {

template <int DT>
__device__ __forceinline__ void vec_update(RowStat& st, const u32x4_t& v) {
  float z[Storage<DT>::kPerVec];
  unpack_vec<DT>(v, z);
  stat_update<Storage<DT>::kPerVec>(st, z);
}

// Streams one row and returns this thread's partial state.  VEC: row base and stride are
// 16-byte aligned.  UNROLL independent 16-byte loads are issued before any is consumed.
template <int NT, int DT, bool VEC, int UNROLL>
__device__ __forceinline__ RowStat row_partial(const void* row, int V) {
  RowStat st = stat_identity();
  const int tid = threadIdx.x;
  if constexpr (VEC) {
    constexpr int E = Storage<DT>::kPerVec;
    const u32x4_t* rv = reinterpret_cast<const u32x4_t*>(row);
    const int nvec = V / E;
    int i = tid;
    for (; i + (UNROLL - 1) * NT < nvec; i += UNROLL * NT) {
      u32x4_t v[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(rv + i + u * NT);
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) vec_update<DT>(st, v[u]);
    }
    for (; i < nvec; i += NT) {
      u32x4_t v = __builtin_nontemporal_load(rv + i);
      vec_update<DT>(st, v);
    }
    const int j = nvec * E + tid;   // ragged tail shorter than one vector
    if (j < V) {
      float z[1] = {load_elt<DT>(row, j)};
      stat_update<1>(st, z);
    }
  } else {
    for (int j = tid; j < V; j += NT) {
      float z[1] = {load_elt<DT>(row, j)};
      stat_update<1>(st, z);
    }
  }
  return st;
}

template <int NT, int DT, bool VEC>
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
  constexpr size_t kEltBytes = Storage<DT>::kBytes;
  const char* row = reinterpret_cast<const char*>(logits) + size_t(t) * size_t(ld) * kEltBytes;
  RowStat st = row_partial<NT, DT, VEC, 4>(row, V);
  st = stat_block_reduce<NT>(st, lds);
  if (threadIdx.x == 0) {
    const float lse = st.m + logf(st.s);
    const float zy = load_elt<DT>(row, y);
    logprob[t] = zy - lse;
    lse_out[t] = lse;
    if (entropy) entropy[t] = lse - st.sz / st.s;
  }
}

template <int NT, int DT, bool VEC>
static void launch_fwd(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                       const uint8_t* row_active, float* logprob, float* entropy, float* lse,
                       int32_t* err_flag, hipStream_t s) {
  hipLaunchKernelGGL((k_logprob_fwd<NT, DT, VEC>), dim3((unsigned)T), dim3(NT), 0, s, logits, T, V, ld,
                     targets, row_active, logprob, entropy, lse, err_flag);
}

template <int DT, bool VEC>
static void dispatch_nt(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                        const uint8_t* row_active, float* logprob, float* entropy, float* lse,
                        int32_t* err_flag, hipStream_t s) {
  // threads per row: one wave for short rows, more as the row grows
  const int per_vec = VEC ? Storage<DT>::kPerVec : 1;
  const int64_t work = (V + per_vec - 1) / per_vec;
  if (work <= 4 * 64) launch_fwd<64, DT, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  else if (work <= 16 * 256) launch_fwd<256, DT, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  else launch_fwd<512, DT, VEC>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
}

// Internal entry used by the loss call when the caller gives no lse.
aero_status logprob_fwd_launch(const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
                               const int32_t* targets, const uint8_t* row_active, float* logprob,
                               float* entropy, float* lse, int32_t* err_flag, hipStream_t s) {
  if (T == 0) return AERO_OK;
  const size_t elt = storage_bytes(dtype);
  const bool vec = (reinterpret_cast<uintptr_t>(logits) % 16 == 0) && ((size_t(ld) * elt) % 16 == 0);
  if (dtype == AERO_BF16) {
    if (vec) dispatch_nt<kBF16, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<kBF16, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  } else if (dtype == AERO_F16) {
    if (vec) dispatch_nt<kF16, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<kF16, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  } else if (dtype == AERO_F8E4M3) {
    if (vec) dispatch_nt<kF8, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<kF8, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  } else {
    if (vec) dispatch_nt<kF32, true>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
    else dispatch_nt<kF32, false>(logits, T, V, ld, targets, row_active, logprob, entropy, lse, err_flag, s);
  }
  return launch_status();
}

}  // namespace aero

extern "C" aero_status aero_logprob_fwd(const void* logits, int32_t dtype, int64_t T, int32_t V, int64_t ld,
                                        const int32_t* targets, const uint8_t* row_active,
                                        float* logprob, float* entropy, float* lse,
                                        int32_t* err_flag, void* stream) {
  if (T < 0 || V < 1 || V > (1 << 24) || ld < V || T > 0x7fffffffLL) return AERO_ERR_SHAPE;
  if (!aero::storage_dtype_ok(dtype)) return AERO_ERR_DTYPE;
  if (T == 0) return AERO_OK;
  if (!logits || !targets || !logprob || !lse) return AERO_ERR_NULL;
  return aero::logprob_fwd_launch(logits, dtype, T, V, ld, targets, row_active, logprob, entropy, lse,
                                  err_flag, aero::as_stream(stream));
}
