// bf16 MFMA GEMM tile for gfx950: D[256 x 256] (fp32) = A[256 x K] * B[256 x K]^T, both
// operands row-major with K contiguous.  One workgroup of 8 waves (2 x 4, two per SIMD) owns
// the tile; each wave accumulates a 128 x 64 sub-tile as 4 x 2 blocks of
// v_mfma_f32_32x32x16_bf16.  Two waves per SIMD let one wave's waits (barrier, LDS latency,
// epilogue arithmetic) hide behind the other's matrix instructions.
//
// Two main loops share the accumulator layout:
//   gemm_tile_dma  operands go HBM -> LDS directly (buffer_load ... lds), ring of five
//                  256 x 32 slices; needs K % 32 == 0 and 16-byte aligned rows
//   gemm_tile      register-staged 256 x 64 slices with explicit predication; any K % 8 == 0
#pragma once
#include "aero_device.h"

namespace aero {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 256;          // tile edge in both output dimensions
constexpr int kGemmNT = 512;        // threads per workgroup (8 waves)
constexpr int kMB = 4, kNB = 2;     // 32 x 32 blocks per wave: 128 rows x 64 columns
constexpr size_t kGemmLdsBytes = 163840;   // all of a CU's LDS: one workgroup per CU

// Position of an accumulator element inside the 256 x 256 tile.
//   block (mb, nb) of wave (wm in 0..1, wn in 0..3); register i of lane l:
//   row = wm*128 + mb*32 + 8*(i/4) + 4*(l/32) + i%4,   col = wn*64 + nb*32 + l%32
__device__ __forceinline__ int acc_row(int wm, int mb, int i, int lane) {
  return wm * 128 + mb * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
}
__device__ __forceinline__ int acc_col(int wn, int nb, int lane) { return wn * 64 + nb * 32 + (lane & 31); }

typedef f32x16_t Acc[kMB][kNB];

__device__ __forceinline__ void acc_zero(Acc& acc) {
#pragma unroll
  for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;
}

// Workgroup id -> tile.  Consecutive hardware workgroup ids go to different XCDs (8 of them,
// each with its own L2), so ids are first regrouped per XCD; inside that order tiles walk
// bands of 8 tile-rows so that concurrently resident workgroups share operand slices in L2.
// xcd_regroup: position of hardware workgroup `pid` (of `nb`) in the per-XCD contiguous order.
__device__ __forceinline__ int xcd_regroup(int pid, int nb) {
  const int q = nb / 8, r = nb % 8, xcd = pid % 8;
  return xcd * q + min(xcd, r) + pid / 8;
}

// npid in [0, tiles_m * tiles_n) -> tile, bands of 8 tile-rows, row index fastest inside a band
__device__ __forceinline__ void tile_of_index(int npid, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int GM = 8;
  const int group_sz = GM * tiles_n;
  const int first_m = (npid / group_sz) * GM;
  const int gm = min(GM, tiles_m - first_m);
  const int within = npid % group_sz;
  tm = first_m + within % gm;
  tn = within / gm;
}

__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
  const int npid = xcd_regroup(blockIdx.x, gridDim.x);
  constexpr int GM = 8;
  const int group_sz = GM * tiles_n;
  const int first_m = (npid / group_sz) * GM;
  const int gm = min(GM, tiles_m - first_m);
  const int within = npid % group_sz;
  tm = first_m + within % gm;
  tn = within / gm;
}

struct Frags {
  bf16x8_t a[kMB], b[kNB];
};

__device__ __forceinline__ void frags_mma(const Frags& f, Acc& acc) {
#pragma unroll
  for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
      acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mb], f.b[nb], acc[mb][nb], 0, 0, 0);
}

// ------------------------------------------------------------------------------------------
// Register-staged loop (fallback): 256 x 64 slices, double buffered, explicit predication.
// ------------------------------------------------------------------------------------------
constexpr int kBK = 64;
constexpr int kSliceElems = kTile * kBK;
constexpr int kVecPerThread = kTile * (kBK / 8) / kGemmNT;   // 4

__device__ __forceinline__ void slice_load(const uint16_t* __restrict__ base, int64_t ld, int row0,
                                           int rows_valid, int k0, int K, u32x4_t (&r)[kVecPerThread]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int v = 0; v < kVecPerThread; ++v) {
    const int idx = tid + v * kGemmNT;
    const int row = row0 + (idx >> 3), k = k0 + ((idx & 7) << 3);
    if (row < rows_valid && k < K)
      r[v] = *reinterpret_cast<const u32x4_t*>(base + int64_t(row) * ld + k);
    else
      r[v] = u32x4_t{0u, 0u, 0u, 0u};
  }
}

// Rows are 128 bytes; rows of equal parity share a 128-byte half of the 256-byte bank line, so
// the chunk index is swizzled with bits 1..3 of the row: 16 consecutive rows -> 16 distinct slots.
__device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * kBK + ((chunk ^ ((row >> 1) & 7)) << 3);
}

__device__ __forceinline__ void slice_store(uint16_t* lds, const u32x4_t (&r)[kVecPerThread]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int v = 0; v < kVecPerThread; ++v) {
    const int idx = tid + v * kGemmNT;
    *reinterpret_cast<u32x4_t*>(lds + lds_off(idx >> 3, idx & 7)) = r[v];
  }
}

__device__ __forceinline__ void slice_mma(const uint16_t* As, const uint16_t* Bs, int wm, int wn, int lane, Acc& acc) {
#pragma unroll
  for (int ks = 0; ks < kBK / 16; ++ks) {
    Frags f;
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
      f.a[mb] = *reinterpret_cast<const bf16x8_t*>(As + lds_off(wm * 128 + mb * 32 + (lane & 31), chunk));
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb)
      f.b[nb] = *reinterpret_cast<const bf16x8_t*>(Bs + lds_off(wn * 64 + nb * 32 + (lane & 31), chunk));
    frags_mma(f, acc);
  }
}

// Full K loop for one tile.  A rows [m0, m0+256) clipped to M, B rows [n0, n0+256) clipped to
// N, columns [0, K).  smem: kGemmLdsBytes.  Ends with a barrier: smem is free afterwards.
__device__ __forceinline__ void gemm_tile(const uint16_t* __restrict__ A, int64_t lda, int M,
                                          const uint16_t* __restrict__ B, int64_t ldb, int N, int K,
                                          int m0, int n0, uint16_t* smem, Acc& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  acc_zero(acc);
  const int nk = (K + kBK - 1) / kBK;
  if (nk == 0) return;
  uint16_t* As[2] = {smem, smem + 2 * kSliceElems};
  uint16_t* Bs[2] = {smem + kSliceElems, smem + 3 * kSliceElems};
  u32x4_t ra[kVecPerThread], rb[kVecPerThread];
  slice_load(A, lda, m0, M, 0, K, ra);
  slice_load(B, ldb, n0, N, 0, K, rb);
  slice_store(As[0], ra);
  slice_store(Bs[0], rb);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
      slice_load(A, lda, m0, M, (kt + 1) * kBK, K, ra);
      slice_load(B, ldb, n0, N, (kt + 1) * kBK, K, rb);
    }
    slice_mma(As[cur], Bs[cur], wm, wn, lane, acc);
    if (more) {
      slice_store(As[cur ^ 1], ra);
      slice_store(Bs[cur ^ 1], rb);
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Direct-to-LDS loop.  buffer_load ... lds moves 16 bytes per lane from HBM/L2 straight into
// LDS (lane l of a wave lands at LDS base + 16 l): no staging registers, no LDS stores, and the
// buffer descriptor's bounds check turns rows past the operand's end into zeros.
//
// Completion of these loads is tracked by hand: every wave issues 4 of them per slice, so
// waiting for "at most 4 x (slices still allowed in flight)" outstanding loads means the oldest
// slice has landed; the barrier then makes every wave's part of it visible.  The compiler does
// not model these dependencies, hence the explicit waits and compiler fences.
// ------------------------------------------------------------------------------------------
constexpr int kDK = 32;                          // K slice of the fast loop
constexpr int kDStages = 5;
constexpr int kDStageElems = 2 * kTile * kDK;    // A then B
static_assert(size_t(kDStages) * kDStageElems * 2 <= kGemmLdsBytes, "ring must fit the LDS budget");
static_assert(size_t(4) * kSliceElems * 2 <= kGemmLdsBytes, "double buffer must fit the LDS budget");

__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const uint16_t* base, int64_t ld, int rows_valid, int K) {
  const int64_t bytes = rows_valid > 0 ? ((int64_t(rows_valid) - 1) * ld + K) * 2 : 0;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, int(bytes), 0x00020000);
}

// 64-byte rows: four rows share a 256-byte bank line, chunk index swizzled with bits 2..3 of the row
__device__ __forceinline__ int dlds_off(int row, int chunk) { return row * kDK + ((chunk ^ ((row >> 2) & 3)) << 3); }

#define AERO_CFENCE() asm volatile("" ::: "memory")

// Wait until at most `slices` slices (4 loads each) of this wave are still in flight, and all of
// its LDS reads have returned.  s_waitcnt takes an immediate: vmcnt in bits 3:0 and 15:14,
// expcnt (unused, 7) in 6:4, lgkmcnt (0) in 11:8.
__device__ __forceinline__ void wait_slices_in_flight(int slices) {
  if (slices >= 3) __builtin_amdgcn_s_waitcnt(0x007C);        // vmcnt(12)
  else if (slices == 2) __builtin_amdgcn_s_waitcnt(0x0078);   // vmcnt(8)
  else if (slices == 1) __builtin_amdgcn_s_waitcnt(0x0074);   // vmcnt(4)
  else __builtin_amdgcn_s_waitcnt(0x0070);                    // vmcnt(0)
}

// wave w fills rows [32 w, 32 w + 32) of both operands: 2 instructions of 16 rows each.
// The whole byte offset travels in the vector offset: the hardware bounds check covers the
// vector offset only, not the scalar one.
__device__ __forceinline__ void dma_issue(__amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, uint32_t voa,
                                          uint32_t vob, uint32_t row_step_a, uint32_t row_step_b, int k0,
                                          uint16_t* stage, int wave) {
  uint16_t* a_dst = stage + wave * 32 * kDK;
  uint16_t* b_dst = stage + kTile * kDK + wave * 32 * kDK;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, a_dst + j * 16 * kDK, 16, voa + uint32_t(k0 * 2) + j * row_step_a, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, b_dst + j * 16 * kDK, 16, vob + uint32_t(k0 * 2) + j * row_step_b, 0, 0, 0);
  }
}

__device__ __forceinline__ void frags_load(Frags& f, const uint16_t* stage, int ks, int wm, int wn, int lane) {
  const uint16_t* As = stage;
  const uint16_t* Bs = stage + kTile * kDK;
  const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
  for (int mb = 0; mb < kMB; ++mb)
    f.a[mb] = *reinterpret_cast<const bf16x8_t*>(As + dlds_off(wm * 128 + mb * 32 + (lane & 31), chunk));
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb)
    f.b[nb] = *reinterpret_cast<const bf16x8_t*>(Bs + dlds_off(wn * 64 + nb * 32 + (lane & 31), chunk));
}

// Slice kt is consumed from registers that were filled one half-slice earlier, so the barrier
// at the top of iteration kt publishes slice kt + 1 (not kt): the fragment reads of the next
// slice overlap the MFMAs of this one.  Slice kt + 4 is issued into the stage slice kt - 1
// used; every wave has finished reading it before it passes this iteration's barrier.
__device__ __forceinline__ void gemm_tile_dma(const uint16_t* __restrict__ A, int64_t lda, int M,
                                              const uint16_t* __restrict__ B, int64_t ldb, int N, int K,
                                              int m0, int n0, uint16_t* smem, Acc& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  acc_zero(acc);
  const int nk = K / kDK;
  if (nk == 0) return;
  const __amdgpu_buffer_rsrc_t ra = operand_rsrc(A, lda, M, K), rb = operand_rsrc(B, ldb, N, K);
  // lane l of an instruction covers row l/4 of its 16 rows, LDS slot l%4; the chunk stored in
  // that slot is slot ^ ((row >> 2) & 3) = (l % 4) ^ (l / 16)
  const uint32_t chunk = uint32_t((lane & 3) ^ (lane >> 4));
  const uint32_t voa = uint32_t((int64_t(m0 + wave * 32 + (lane >> 2)) * lda) * 2) + chunk * 16;
  const uint32_t vob = uint32_t((int64_t(n0 + wave * 32 + (lane >> 2)) * ldb) * 2) + chunk * 16;
  const uint32_t step_a = uint32_t(16 * lda * 2), step_b = uint32_t(16 * ldb * 2);
#pragma unroll
  for (int s = 0; s < kDStages - 1; ++s)
    if (s < nk) dma_issue(ra, rb, voa, vob, step_a, step_b, s * kDK, smem + s * kDStageElems, wave);
  constexpr int kAhead = kDStages - 1;             // slices issued ahead of the one being consumed
  wait_slices_in_flight(min(nk, kAhead) - 1);      // slice 0 has landed
  AERO_CFENCE();
  __builtin_amdgcn_s_barrier();
  AERO_CFENCE();
  Frags f0, f1;
  frags_load(f0, smem, 0, wm, wn, lane);
  for (int kt = 0; kt < nk; ++kt) {
    // slices 0 .. kt + 1 have landed; the later ones already issued may stay in flight
    wait_slices_in_flight(max(0, min(nk, kt + kAhead) - kt - 2));
    AERO_CFENCE();
    __builtin_amdgcn_s_barrier();
    AERO_CFENCE();
    if (kt + kDStages - 1 < nk)
      dma_issue(ra, rb, voa, vob, step_a, step_b, (kt + kDStages - 1) * kDK,
                smem + ((kt + kDStages - 1) % kDStages) * kDStageElems, wave);
    frags_load(f1, smem + (kt % kDStages) * kDStageElems, 1, wm, wn, lane);
    frags_mma(f0, acc);
    // after the last slice this reads a stage nobody writes any more; the values are unused
    frags_load(f0, smem + ((kt + 1) % kDStages) * kDStageElems, 0, wm, wn, lane);
    frags_mma(f1, acc);
  }
  __syncthreads();
}

// Picks the fast loop when its preconditions hold (uniform over the launch).
__device__ __forceinline__ void gemm_tile_auto(const uint16_t* __restrict__ A, int64_t lda, int M,
                                               const uint16_t* __restrict__ B, int64_t ldb, int N, int K,
                                               int m0, int n0, uint16_t* smem, Acc& acc) {
  const bool fast = (K % kDK == 0) && (lda % 8 == 0) && (ldb % 8 == 0) &&
                    (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (reinterpret_cast<uintptr_t>(B) % 16 == 0) &&
                    ((int64_t(M) - 1) * lda + K) < (int64_t(1) << 31) && ((int64_t(N) - 1) * ldb + K) < (int64_t(1) << 31);
  if (fast) gemm_tile_dma(A, lda, M, B, ldb, N, K, m0, n0, smem, acc);
  else gemm_tile(A, lda, M, B, ldb, N, K, m0, n0, smem, acc);
}

}  // namespace aero
