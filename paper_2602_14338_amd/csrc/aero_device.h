// Device-side helpers shared by the kernels: bf16 packing, wave64 reductions,
// the running (max, sum-exp, sum-exp-times-logit) state of a softmax row.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/aero.h"

namespace aero {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kWave = 64;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // one 16-byte global access

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// two floats -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  bf16x2_t b = __builtin_convertvector(f, bf16x2_t);
  return *reinterpret_cast<uint32_t*>(&b);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float x) {
  return uint16_t(pack_bf16x2(x, 0.f) & 0xffffu);
}

// IEEE binary16 storage: widening is exact, narrowing rounds to nearest even (subnormals kept).
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float f16_to_f32(uint16_t b) {
  _Float16 h;
  __builtin_memcpy(&h, &b, 2);
  return float(h);
}
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  f32x2_t f = {lo, hi};
  f16x2_t h = __builtin_convertvector(f, f16x2_t);
  uint32_t w;
  __builtin_memcpy(&w, &h, 4);
  return w;
}
__device__ __forceinline__ uint16_t f32_to_f16(float x) { return uint16_t(pack_f16x2(x, 0.f) & 0xffffu); }

// 8-bit float storage, 4 exponent and 3 mantissa bits, no infinities (largest finite value 448): widening is
// exact; narrowing rounds to nearest even, keeps subnormals (multiples of 2^-9) and saturates beyond +-448.
__device__ __forceinline__ float f8_to_f32(uint8_t b) { return __builtin_amdgcn_cvt_f32_fp8(int(b), 0); }
__device__ __forceinline__ uint32_t pack_f8x4(float a, float b, float c, float d) {
  constexpr float kMax = 448.f;
  a = __builtin_amdgcn_fmed3f(a, -kMax, kMax);
  b = __builtin_amdgcn_fmed3f(b, -kMax, kMax);
  c = __builtin_amdgcn_fmed3f(c, -kMax, kMax);
  d = __builtin_amdgcn_fmed3f(d, -kMax, kMax);
  int p = 0;
  p = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, p, false);   // low half of the word
  p = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, p, true);    // high half
  return uint32_t(p);
}
__device__ __forceinline__ uint8_t f32_to_f8(float x) { return uint8_t(pack_f8x4(x, 0.f, 0.f, 0.f) & 0xffu); }

// Storage type tags (the values of the public dtype codes) and what depends on them.
constexpr int kF32 = AERO_F32, kBF16 = AERO_BF16, kF16 = AERO_F16, kF8 = AERO_F8E4M3;
template <int DT> struct Storage {
  static constexpr int kBytes = DT == kF32 ? 4 : DT == kF8 ? 1 : 2;
  static constexpr int kPerVec = 16 / kBytes;   // elements per 16-byte vector
};
inline bool storage_dtype_ok(int32_t dtype) {
  return dtype == AERO_BF16 || dtype == AERO_F32 || dtype == AERO_F16 || dtype == AERO_F8E4M3;
}
inline size_t storage_bytes(int32_t dtype) { return dtype == AERO_F32 ? 4 : dtype == AERO_F8E4M3 ? 1 : 2; }
template <int DT> __device__ __forceinline__ float load_elt(const void* row, int64_t j) {
  if constexpr (DT == kBF16) return bf16_to_f32(reinterpret_cast<const uint16_t*>(row)[j]);
  else if constexpr (DT == kF16) return f16_to_f32(reinterpret_cast<const uint16_t*>(row)[j]);
  else if constexpr (DT == kF8) return f8_to_f32(reinterpret_cast<const uint8_t*>(row)[j]);
  else return reinterpret_cast<const float*>(row)[j];
}
template <int DT> __device__ __forceinline__ void store_elt(void* row, int64_t j, float x) {
  if constexpr (DT == kBF16) reinterpret_cast<uint16_t*>(row)[j] = f32_to_bf16(x);
  else if constexpr (DT == kF16) reinterpret_cast<uint16_t*>(row)[j] = f32_to_f16(x);
  else if constexpr (DT == kF8) reinterpret_cast<uint8_t*>(row)[j] = f32_to_f8(x);
  else reinterpret_cast<float*>(row)[j] = x;
}

__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Softmax row state relative to an offset m (any m close enough to the row maximum that
// nothing overflows): s = sum exp(z - m), sz = sum exp(z - m) z.
struct RowStat {
  float m, s, sz;
};

__device__ __forceinline__ RowStat stat_identity() { return RowStat{-INFINITY, 0.f, 0.f}; }

__device__ __forceinline__ RowStat stat_merge(RowStat a, RowStat b) {
  float M = fmaxf(a.m, b.m);
  float fa = (a.m == M) ? 1.f : exp2_fast((a.m - M) * kLog2e);
  float fb = (b.m == M) ? 1.f : exp2_fast((b.m - M) * kLog2e);
  return RowStat{M, a.s * fa + b.s * fb, a.sz * fa + b.sz * fb};
}

__device__ __forceinline__ RowStat stat_shfl_xor(RowStat a, int mask) {
  return RowStat{__shfl_xor(a.m, mask, kWave), __shfl_xor(a.s, mask, kWave), __shfl_xor(a.sz, mask, kWave)};
}

__device__ __forceinline__ RowStat stat_wave_reduce(RowStat a) {
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) a = stat_merge(a, stat_shfl_xor(a, off));
  return a;
}

// Workgroup-wide merge; every thread gets the result.  NT = threads per workgroup.
template <int NT>
__device__ __forceinline__ RowStat stat_block_reduce(RowStat a, RowStat* lds /*[NT/64]*/) {
  a = stat_wave_reduce(a);
  if constexpr (NT > kWave) {
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    if (lane == 0) lds[wave] = a;
    __syncthreads();
    RowStat r = lds[0];
#pragma unroll
    for (int w = 1; w < NT / kWave; ++w) r = stat_merge(r, lds[w]);
    a = r;
  }
  return a;
}

// Fold N logits into a thread's running state.  The offset m is only moved when a value
// exceeds it by more than kLazy nats, so the rescale is rare and exp(z - m) stays below
// e^kLazy; sums of 2^24 such terms stay far inside fp32 range.
constexpr float kLazy = 12.0f;

template <int N>
__device__ __forceinline__ void stat_update(RowStat& st, const float (&z)[N]) {
  float vm = z[0];
  if constexpr (N >= 3) {
#pragma unroll
    for (int k = 1; k + 1 < N; k += 2) vm = max3(vm, z[k], z[k + 1]);
    if constexpr (N % 2 == 0) vm = fmaxf(vm, z[N - 1]);
  } else if constexpr (N == 2) {
    vm = fmaxf(vm, z[1]);
  }
  // also taken on first use (m = -inf).  The wave-uniform test in front keeps the compiler from
  // turning the rare rescale into always-executed predicated code (about two extra vector
  // instructions per logit in kernels whose vector ALUs are close to saturated).
  const bool grow = vm > st.m + kLazy;
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
    asm volatile("" ::: "memory");   // a side effect: the block cannot be if-converted
    if (grow) {
      float f = (st.m == -INFINITY) ? 0.f : exp2_fast((st.m - vm) * kLog2e);
      st.s *= f;
      st.sz *= f;
      st.m = vm;
    }
  }
  const float c = -st.m * kLog2e;
#pragma unroll
  for (int k = 0; k < N; ++k) {
    float e = exp2_fast(fmaf(z[k], kLog2e, c));
    st.s += e;
    st.sz = fmaf(e, z[k], st.sz);
  }
}

__device__ __forceinline__ void unpack8(const u32x4_t& v, float (&z)[8]) {
  z[0] = bf16_lo(v.x); z[1] = bf16_hi(v.x);
  z[2] = bf16_lo(v.y); z[3] = bf16_hi(v.y);
  z[4] = bf16_lo(v.z); z[5] = bf16_hi(v.z);
  z[6] = bf16_lo(v.w); z[7] = bf16_hi(v.w);
}

__device__ __forceinline__ void unpack8_f16(const u32x4_t& v, float (&z)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    f16x2_t h;
    __builtin_memcpy(&h, &w[k], 4);
    z[2 * k] = float(h.x);
    z[2 * k + 1] = float(h.y);
  }
}

__device__ __forceinline__ void unpack16_f8(const u32x4_t& v, float (&z)[16]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f32x2_t lo = __builtin_amdgcn_cvt_pk_f32_fp8(int(w[k]), false);
    const f32x2_t hi = __builtin_amdgcn_cvt_pk_f32_fp8(int(w[k]), true);
    z[4 * k] = lo.x; z[4 * k + 1] = lo.y;
    z[4 * k + 2] = hi.x; z[4 * k + 3] = hi.y;
  }
}

// One 16-byte vector of stored logits -> floats (16 for the 8-bit type, 8 for the 2-byte types, 4 for fp32) and back.
template <int DT> __device__ __forceinline__ void unpack_vec(const u32x4_t& v, float (&z)[Storage<DT>::kPerVec]) {
  if constexpr (DT == kBF16) unpack8(v, z);
  else if constexpr (DT == kF16) unpack8_f16(v, z);
  else if constexpr (DT == kF8) unpack16_f8(v, z);
  else {
    z[0] = __uint_as_float(v.x); z[1] = __uint_as_float(v.y);
    z[2] = __uint_as_float(v.z); z[3] = __uint_as_float(v.w);
  }
}
template <int DT> __device__ __forceinline__ u32x4_t pack_vec(const float (&d)[Storage<DT>::kPerVec]) {
  u32x4_t o;
  if constexpr (DT == kBF16) {
    o.x = pack_bf16x2(d[0], d[1]); o.y = pack_bf16x2(d[2], d[3]);
    o.z = pack_bf16x2(d[4], d[5]); o.w = pack_bf16x2(d[6], d[7]);
  } else if constexpr (DT == kF16) {
    o.x = pack_f16x2(d[0], d[1]); o.y = pack_f16x2(d[2], d[3]);
    o.z = pack_f16x2(d[4], d[5]); o.w = pack_f16x2(d[6], d[7]);
  } else if constexpr (DT == kF8) {
    o.x = pack_f8x4(d[0], d[1], d[2], d[3]);     o.y = pack_f8x4(d[4], d[5], d[6], d[7]);
    o.z = pack_f8x4(d[8], d[9], d[10], d[11]);   o.w = pack_f8x4(d[12], d[13], d[14], d[15]);
  } else {
    o.x = __float_as_uint(d[0]); o.y = __float_as_uint(d[1]);
    o.z = __float_as_uint(d[2]); o.w = __float_as_uint(d[3]);
  }
  return o;
}

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

inline aero_status launch_status() {
  return hipGetLastError() == hipSuccess ? AERO_OK : AERO_ERR_HIP;
}

}  // namespace aero
