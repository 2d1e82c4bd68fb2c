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

}  // namespace aero
