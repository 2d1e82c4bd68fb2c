// bf16 MFMA GEMM tile for gfx950: D[256 x 256] (fp32) = A[256 x K] * B[256 x K]^T, both
// operands row-major with K contiguous.  One workgroup of 4 waves (2 x 2) owns the tile; each
// wave accumulates a 128 x 128 sub-tile as 4 x 4 blocks of v_mfma_f32_32x32x16_bf16.
//
// Operands are staged HBM -> registers -> LDS in 256 x 64 slices, double buffered (one
// barrier per slice); the 16-byte chunks of each LDS row are XOR-swizzled with the row index
// so that the 128-bit fragment reads of 16 consecutive rows hit distinct banks.
#pragma once
#include "aero_device.h"

namespace aero {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 256;          // tile edge in both output dimensions
constexpr int kBK = 64;             // K slice
constexpr int kGemmNT = 256;        // threads per workgroup
constexpr int kSliceElems = kTile * kBK;
constexpr size_t kGemmLdsBytes = size_t(2) * 2 * kSliceElems * sizeof(uint16_t);   // 128 KiB

// Position of an accumulator element inside the 256 x 256 tile.
//   block (mb, nb) of wave (wm, wn); register i of lane l:
//   row = wm*128 + mb*32 + 8*(i/4) + 4*(l/32) + i%4,   col = wn*128 + nb*32 + l%32
__device__ __forceinline__ int acc_row(int wm, int mb, int i, int lane) {
  return wm * 128 + mb * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
}
__device__ __forceinline__ int acc_col(int wn, int nb, int lane) { return wn * 128 + nb * 32 + (lane & 31); }

// Workgroup id -> tile.  Consecutive hardware workgroup ids go to different XCDs (8 of them,
// each with its own L2), so ids are first regrouped per XCD; inside that order tiles walk
// bands of 8 tile-rows so that concurrently resident workgroups share operand slices in L2.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
  const int nb = gridDim.x, pid = blockIdx.x;
  const int q = nb / 8, r = nb % 8, xcd = pid % 8;
  const int npid = xcd * q + min(xcd, r) + pid / 8;
  constexpr int GM = 8;
  const int group_sz = GM * tiles_n;
  const int first_m = (npid / group_sz) * GM;
  const int gm = min(GM, tiles_m - first_m);
  const int within = npid % group_sz;
  tm = first_m + within % gm;
  tn = within / gm;
}

// 256 x 64 slice of a row-major operand -> 8 x 16 bytes per thread.  Rows >= rows_valid and
// columns >= K read as zero, so ragged edges contribute nothing.
__device__ __forceinline__ void slice_load(const uint16_t* __restrict__ base, int64_t ld, int row0,
                                           int rows_valid, int k0, int K, u32x4_t (&r)[8]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
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

__device__ __forceinline__ void slice_store(uint16_t* lds, const u32x4_t (&r)[8]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int v = 0; v < 8; ++v) {
    const int idx = tid + v * kGemmNT;
    *reinterpret_cast<u32x4_t*>(lds + lds_off(idx >> 3, idx & 7)) = r[v];
  }
}

__device__ __forceinline__ void slice_mma(const uint16_t* As, const uint16_t* Bs, int wm, int wn, int lane,
                                          f32x16_t (&acc)[4][4]) {
#pragma unroll
  for (int ks = 0; ks < kBK / 16; ++ks) {
    bf16x8_t a[4], b[4];
    const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
      const int row = wm * 128 + mb * 32 + (lane & 31);
      a[mb] = *reinterpret_cast<const bf16x8_t*>(As + lds_off(row, chunk));
    }
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int row = wn * 128 + nb * 32 + (lane & 31);
      b[nb] = *reinterpret_cast<const bf16x8_t*>(Bs + lds_off(row, chunk));
    }
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], b[nb], acc[mb][nb], 0, 0, 0);
  }
}

// Full K loop for one tile.  A rows [m0, m0+256) clipped to M, B rows [n0, n0+256) clipped to
// N, columns [0, K).  smem: kGemmLdsBytes.  Ends with a barrier: smem is free afterwards.
__device__ __forceinline__ void gemm_tile(const uint16_t* __restrict__ A, int64_t lda, int M,
                                          const uint16_t* __restrict__ B, int64_t ldb, int N, int K,
                                          int m0, int n0, uint16_t* smem, f32x16_t (&acc)[4][4]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;
  const int nk = (K + kBK - 1) / kBK;
  if (nk == 0) return;
  uint16_t* As[2] = {smem, smem + 2 * kSliceElems};
  uint16_t* Bs[2] = {smem + kSliceElems, smem + 3 * kSliceElems};
  u32x4_t ra[8], rb[8];
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
// Fast main loop: operands go HBM -> LDS directly (buffer_load ... lds, 16 bytes per lane,
// lane l of a wave lands at LDS base + 16 l), no staging registers and no LDS stores.
// Slices are 256 x 32 (64-byte rows), four of them in flight in a ring of four stages;
// the hardware bounds check of the buffer descriptor turns rows past the operand's end into
// zeros.  Needs K % 32 == 0 and 16-byte aligned operands; callers fall back to gemm_tile
// otherwise.
//
// LDS-DMA completion is tracked by hand: every wave issues 8 loads per slice, so waiting for
// "at most 8 x (slices still allowed in flight)" outstanding loads means the oldest slice has
// landed; the barrier then makes every wave's part of it visible.  The compiler does not
// model these dependencies, hence the explicit waits and compiler fences.
// ------------------------------------------------------------------------------------------
constexpr int kDK = 32;                          // K slice of the fast loop
constexpr int kDStages = 4;
constexpr int kDStageElems = 2 * kTile * kDK;    // A then B
static_assert(size_t(kDStages) * kDStageElems * 2 <= kGemmLdsBytes, "ring must fit the LDS budget");

__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const uint16_t* base, int64_t ld, int rows_valid, int K) {
  const int64_t bytes = rows_valid > 0 ? ((int64_t(rows_valid) - 1) * ld + K) * 2 : 0;
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, int(bytes), 0x00020000);
}

// 64-byte rows: four rows share a 256-byte bank line, chunk index swizzled with bits 2..3 of the row
__device__ __forceinline__ int dlds_off(int row, int chunk) { return row * kDK + ((chunk ^ ((row >> 2) & 3)) << 3); }

#define AERO_WAIT_VM16() __builtin_amdgcn_s_waitcnt(0x4070)   /* vmcnt(16) lgkmcnt(0) */
#define AERO_WAIT_VM8() __builtin_amdgcn_s_waitcnt(0x0078)    /* vmcnt(8)  lgkmcnt(0) */
#define AERO_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0x0070)    /* vmcnt(0)  lgkmcnt(0) */
#define AERO_CFENCE() asm volatile("" ::: "memory")

__device__ __forceinline__ void dma_issue(__amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, uint32_t voa,
                                          uint32_t vob, uint32_t row_step_a, uint32_t row_step_b, int k0,
                                          uint16_t* stage, int wave) {
  // wave w fills rows [64 w, 64 w + 64) of both operands: 4 instructions of 16 rows each
  uint16_t* a_dst = stage + wave * 64 * kDK;
  uint16_t* b_dst = stage + kTile * kDK + wave * 64 * kDK;
  // the whole byte offset travels in the vector offset: the hardware bounds check covers the
  // vector offset only, not the scalar one
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, a_dst + j * 16 * kDK, 16, voa + uint32_t(k0 * 2) + j * row_step_a, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, b_dst + j * 16 * kDK, 16, vob + uint32_t(k0 * 2) + j * row_step_b, 0, 0, 0);
  }
}

struct Frags {
  bf16x8_t a[4], b[4];
};

__device__ __forceinline__ void frags_load(Frags& f, const uint16_t* stage, int ks, int wm, int wn, int lane) {
  const uint16_t* As = stage;
  const uint16_t* Bs = stage + kTile * kDK;
  const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
    f.a[mb] = *reinterpret_cast<const bf16x8_t*>(As + dlds_off(wm * 128 + mb * 32 + (lane & 31), chunk));
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
    f.b[nb] = *reinterpret_cast<const bf16x8_t*>(Bs + dlds_off(wn * 128 + nb * 32 + (lane & 31), chunk));
}

__device__ __forceinline__ void frags_mma(const Frags& f, f32x16_t (&acc)[4][4]) {
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
      acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[mb], f.b[nb], acc[mb][nb], 0, 0, 0);
}

// Slice kt is consumed from registers that were filled one half-slice earlier, so the barrier
// at the top of iteration kt publishes slice kt + 1 (not kt): the fragment reads of the next
// slice overlap the MFMAs of this one.  Slice kt + 3 is issued into the stage slice kt - 1
// used; every wave has finished reading it before it passes this iteration's barrier.
__device__ __forceinline__ void gemm_tile_dma(const uint16_t* __restrict__ A, int64_t lda, int M,
                                              const uint16_t* __restrict__ B, int64_t ldb, int N, int K,
                                              int m0, int n0, uint16_t* smem, f32x16_t (&acc)[4][4]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int mb = 0; mb < 4; ++mb)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;
  const int nk = K / kDK;
  if (nk == 0) return;
  const __amdgpu_buffer_rsrc_t ra = operand_rsrc(A, lda, M, K), rb = operand_rsrc(B, ldb, N, K);
  // lane l of an instruction covers row l/4 of its 16 rows, LDS slot l%4; the chunk stored in
  // that slot is slot ^ ((row >> 2) & 3) = (l % 4) ^ (l / 16)
  const uint32_t chunk = uint32_t((lane & 3) ^ (lane >> 4));
  const uint32_t voa = uint32_t((int64_t(m0 + wave * 64 + (lane >> 2)) * lda) * 2) + chunk * 16;
  const uint32_t vob = uint32_t((int64_t(n0 + wave * 64 + (lane >> 2)) * ldb) * 2) + chunk * 16;
  const uint32_t step_a = uint32_t(16 * lda * 2), step_b = uint32_t(16 * ldb * 2);
#pragma unroll
  for (int s = 0; s < kDStages - 1; ++s)
    if (s < nk) dma_issue(ra, rb, voa, vob, step_a, step_b, s * kDK, smem + s * kDStageElems, wave);
  if (nk >= 3) AERO_WAIT_VM16();
  else if (nk == 2) AERO_WAIT_VM8();
  else AERO_WAIT_VM0();
  AERO_CFENCE();
  __builtin_amdgcn_s_barrier();
  AERO_CFENCE();
  Frags f0, f1;
  frags_load(f0, smem, 0, wm, wn, lane);
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 2 < nk) AERO_WAIT_VM8();   // slice kt + 1 has landed, kt + 2 may be in flight
    else AERO_WAIT_VM0();
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
                                               int m0, int n0, uint16_t* smem, f32x16_t (&acc)[4][4]) {
  const bool fast = (K % kDK == 0) && (lda % 8 == 0) && (ldb % 8 == 0) &&
                    (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (reinterpret_cast<uintptr_t>(B) % 16 == 0) &&
                    ((int64_t(M) - 1) * lda + K) < (int64_t(1) << 31) && ((int64_t(N) - 1) * ldb + K) < (int64_t(1) << 31);
  if (fast) gemm_tile_dma(A, lda, M, B, ldb, N, K, m0, n0, smem, acc);
  else gemm_tile(A, lda, M, B, ldb, N, K, m0, n0, smem, acc);
}

}  // namespace aero
