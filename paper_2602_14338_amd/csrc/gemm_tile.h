// bf16 MFMA GEMM tile for gfx950: D[256 x 256] (fp32) = A[256 x K] * B[256 x K]^T, both
// operands row-major with K contiguous.  One workgroup of 8 waves (2 x 4, two per SIMD) owns
// the tile; each wave accumulates a 128 x 64 sub-tile as 4 x 2 blocks of
// v_mfma_f32_32x32x16_bf16.  Two waves per SIMD let one wave's waits (barrier, LDS latency,
// epilogue arithmetic) hide behind the other's matrix instructions.
//
// Two main loops share the accumulator layout:
//   gemm_tile_dma  operands go HBM -> LDS directly (buffer_load ... lds), two stages of
//                  256 x 64 slices, L2 warmed two slices ahead; needs K % 64 == 0 and
//                  16-byte aligned rows
//   gemm_tile      register-staged 256 x 64 slices with explicit predication; any K % 8 == 0
#pragma once
#include "aero_device.h"

namespace aero {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kTile = 256;          // tile edge in both output dimensions
constexpr int kGemmNT = 512;        // threads per workgroup (8 waves)
constexpr int kMB = 4, kNB = 2;     // 32 x 32 blocks per wave: 128 rows x 64 columns
constexpr size_t kGemmStageBytes = 131072;  // two stages of (256 + 256) x 64 bf16
constexpr size_t kWarmSinkOff = 135168;     // past the stages (128 KB) and the largest epilogue staging area (256 x 256 bf16)
constexpr size_t kGemmLdsBytes = kWarmSinkOff + 2048;   // + a 256-byte sink per wave for the warm-up loads

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

// The same regrouping in whole columns of a band: the n positions of a launch are cut into units
// of 8 consecutive positions (one column of 8 tile rows), every XCD gets a contiguous run of
// whole units (run lengths differ by at most one unit), so that the workgroups resident on an
// XCD always cover whole columns, whatever n is.  The launch grid is xcd_grid(n) >= n workgroups;
// the surplus ones get -1 and leave.
inline int xcd_grid(int n) { return 64 * (((n + 7) / 8 + 7) / 8); }
__device__ __forceinline__ int xcd_position(int pid, int n) {
  const int units = (n + 7) / 8, q = units / 8, r = units % 8;
  const int xcd = pid % 8, local = pid / 8;
  const int ul = local / 8;
  if (ul >= q + (xcd < r ? 1 : 0)) return -1;
  const int pos = (xcd * q + min(xcd, r) + ul) * 8 + local % 8;
  return pos < n ? pos : -1;
}

// tile0: position in the tile order of this launch's first tile, n: tiles of this launch (a
// kernel's tiles may be spread over several launches).  False: a surplus workgroup.
__device__ __forceinline__ bool tile_of_block(int tiles_m, int tiles_n, int tile0, int n, int& tm, int& tn) {
  const int pos = xcd_position(blockIdx.x, n);
  if (pos < 0) return false;
  const int npid = tile0 + pos;
  constexpr int GM = 8;
  const int group_sz = GM * tiles_n;
  const int first_m = (npid / group_sz) * GM;
  const int gm = min(GM, tiles_m - first_m);
  const int within = npid % group_sz;
  tm = first_m + within % gm;
  tn = within / gm;
  return true;
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
static_assert(size_t(4) * kSliceElems * 2 <= kGemmStageBytes, "double buffer must fit the LDS budget");
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
// buffer descriptor's bounds check turns rows past the operand's end into zeros.  Slices are
// 256 x 64: every row contributes one full 128-byte line per slice (32-wide slices fetch half
// lines and lose a tenth of the throughput), two stages of 64 KB.
//
// Completion of these loads is tracked by hand: vmcnt(0) at the top of an iteration means this
// wave's part of the slice has landed, the barrier then makes every wave's part visible and
// also guarantees that the other stage is no longer being read.  The compiler does not model
// these dependencies, hence the explicit waits and compiler fences.
// ------------------------------------------------------------------------------------------
constexpr int kDK = kBK;                         // K slice of the fast loop
constexpr int kDStageElems = 2 * kTile * kDK;    // A then B
static_assert(size_t(2) * kDStageElems * 2 <= kGemmStageBytes, "two stages must fit the LDS budget");

// An operand of the fast loop: rows of 64-wide K slices.  Element (row, k) lives at
//   base + (k / 64) * kstep + row * ld + k % 64
//   row-major [rows, K]:            ld = row pitch, kstep = 64
//   K-slab layout [K/64][rows][64]: ld = 64,        kstep = rows * 64  (a 256-row slice is one
//                                   contiguous 32 KB block: the layout of the library's own
//                                   intermediate operands)
// bytes bounds the buffer: loads past it return zeros.
struct DmaOperand {
  const uint16_t* base;
  int64_t ld, kstep, bytes;
};
__device__ __forceinline__ DmaOperand operand_row_major(const uint16_t* base, int64_t ld, int rows_valid, int K) {
  return DmaOperand{base, ld, kDK, rows_valid > 0 ? ((int64_t(rows_valid) - 1) * ld + K) * 2 : 0};
}
__device__ __forceinline__ DmaOperand operand_slabs(const uint16_t* base, int64_t rows, int K) {
  return DmaOperand{base, kDK, rows * kDK, int64_t(K / kDK) * rows * kDK * 2};
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t operand_rsrc(const DmaOperand& o) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(o.base), 0, int(o.bytes), 0x00020000);
}

#define AERO_CFENCE() asm volatile("" ::: "memory")

// Per-lane byte offsets of the DMA loads of one operand.  Wave w fills rows [32 w, 32 w + 32)
// with 4 instructions of 8 rows; lane l covers row l/8 of those 8 and LDS slot l%8, and the
// chunk that belongs in that slot is slot ^ ((row >> 1) & 7) with row = 32 w + 8 j + l/8, i.e.
// (l % 8) ^ ((4 j + l / 16) & 7): one offset for even j, one for odd j.
struct DmaLane {
  uint32_t even, odd, row_step, k_step;
};
__device__ __forceinline__ DmaLane dma_lane(int row0, const DmaOperand& o, int wave, int lane) {
  const uint32_t row = uint32_t((int64_t(row0 + wave * 32 + (lane >> 3)) * o.ld) * 2);
  const uint32_t c0 = uint32_t((lane & 7) ^ ((lane >> 4) & 7)), c1 = uint32_t((lane & 7) ^ ((4 + (lane >> 4)) & 7));
  return DmaLane{row + c0 * 16, row + c1 * 16, uint32_t(8 * o.ld * 2), uint32_t(o.kstep * 2)};
}

// The whole byte offset travels in the vector offset: the hardware bounds check covers the
// vector offset only, not the scalar one.
__device__ __forceinline__ void dma_issue(__amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, const DmaLane& la,
                                          const DmaLane& lb, int kt, uint16_t* stage, int wave) {
  uint16_t* a_dst = stage + wave * 32 * kDK;
  uint16_t* b_dst = stage + kTile * kDK + wave * 32 * kDK;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, a_dst + j * 8 * kDK, 16,
                                             ((j & 1) ? la.odd : la.even) + uint32_t(kt) * la.k_step + j * la.row_step, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, b_dst + j * 8 * kDK, 16,
                                             ((j & 1) ? lb.odd : lb.even) + uint32_t(kt) * lb.k_step + j * lb.row_step, 0, 0, 0);
  }
}

__device__ __forceinline__ void frags_load(Frags& f, const uint16_t* stage, int ks, int wm, int wn, int lane) {
  const uint16_t* As = stage;
  const uint16_t* Bs = stage + kTile * kDK;
  const int chunk = ks * 2 + (lane >> 5);
#pragma unroll
  for (int mb = 0; mb < kMB; ++mb)
    f.a[mb] = *reinterpret_cast<const bf16x8_t*>(As + lds_off(wm * 128 + mb * 32 + (lane & 31), chunk));
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb)
    f.b[nb] = *reinterpret_cast<const bf16x8_t*>(Bs + lds_off(wn * 64 + nb * 32 + (lane & 31), chunk));
}

// WARM: L2 warm-up two slices ahead (see below); a few per cent on the contractions whose
// operands come from large read-only arrays, a loss on the split-K dhidden contraction.
template <bool WARM>
__device__ __forceinline__ void gemm_tile_dma(const DmaOperand& A, const DmaOperand& B, int K, int m0, int n0,
                                              uint16_t* smem, Acc& acc) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  acc_zero(acc);
  const int nk = K / kDK;
  if (nk == 0) return;
  const __amdgpu_buffer_rsrc_t ra = operand_rsrc(A), rb = operand_rsrc(B);
  const DmaLane la = dma_lane(m0, A, wave, lane), lb = dma_lane(n0, B, wave, lane);
  dma_issue(ra, rb, la, lb, 0, smem, wave);
  // L2 warm-up.  A fifth of a slice's lines miss L2 (the 32 workgroups resident on an XCD form an
  // 8 x 4 block of tiles: 12 operand slices for 32 tiles), and loads return in order, so one late
  // line holds back everything queued behind it.  Each slice is therefore touched two slices
  // early with one 4-byte load per 128-byte line (sunk into a scratch corner of LDS), the lines
  // shared out over the workgroups that will read them: wave 0 takes a quarter of the A rows
  // (which quarter: by tile column), wave 4 an eighth of the B rows (by tile row).  The touch is
  // issued late in the slice, when every wave's requests for the next slice are already queued
  // ahead of it, and it may stay in flight across the next barrier (vmcnt(1)).
  constexpr int kWarmAhead = 2;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);   // wave-uniform: the descriptor stays scalar
  const bool warm_a = wave_u < 4, warm_wave = WARM && (wave_u & 3) == 0;
  const __amdgpu_buffer_rsrc_t rw = warm_a ? ra : rb;
  const int warm_row = warm_a ? m0 + ((n0 / kTile) & 3) * 64 + lane : n0 + ((m0 / kTile) & 7) * 32 + (lane & 31);
  const uint32_t warm_off = uint32_t(int64_t(warm_row) * (warm_a ? A.ld : B.ld) * 2) + (warm_a ? 0u : uint32_t(lane >> 5) * 64u);
  const uint32_t warm_kstep = uint32_t((warm_a ? A.kstep : B.kstep) * 2);
  uint16_t* const warm_sink = smem + kWarmSinkOff / 2 + wave * 128;
  // One iteration = one 64-wide slice = four 16-wide steps of 8 MFMAs per wave.  The order is
  // pinned with scheduling barriers: both fragment sets of the first two steps are read up
  // front, the next slice is requested only after the first MFMA group (issuing the 8 loads
  // right after the barrier would hold back every wave's first MFMAs: measured 8 % slower),
  // and the fragment reads of steps 2 and 3 are interleaved one-to-one with MFMAs.
  // warm: touch slice kt + kWarmAhead; warm_pending: the previous slice issued a touch.
  auto slice = [&](int kt, bool prefetch, bool warm, bool warm_pending) {
    // slice kt landed (the youngest load may be a touch: loads return in order), own LDS reads done
    if (warm_pending && warm_wave) __builtin_amdgcn_s_waitcnt(0x0071);   // vmcnt(1) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0070);                             // vmcnt(0) lgkmcnt(0)
    AERO_CFENCE();
    __builtin_amdgcn_s_barrier();
    AERO_CFENCE();
    const uint16_t* st = smem + (kt & 1) * kDStageElems;
    Frags f0, f1;
    frags_load(f0, st, 0, wm, wn, lane);
    frags_load(f1, st, 1, wm, wn, lane);
    frags_mma(f0, acc);
    if (prefetch) dma_issue(ra, rb, la, lb, kt + 1, smem + ((kt + 1) & 1) * kDStageElems, wave);
    frags_load(f0, st, 2, wm, wn, lane);
    frags_mma(f1, acc);
    frags_load(f1, st, 3, wm, wn, lane);
    frags_mma(f0, acc);
    constexpr int kMfma = 0x008, kVmemRd = 0x020, kDsRd = 0x100;
    constexpr int kFragReads = kMB + kNB, kMfmas = kMB * kNB;
    __builtin_amdgcn_sched_group_barrier(kDsRd, 2 * kFragReads, 0);
    __builtin_amdgcn_sched_group_barrier(kMfma, kMfmas, 0);
    if (prefetch) __builtin_amdgcn_sched_group_barrier(kVmemRd, 8, 0);
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
#pragma unroll
      for (int r = 0; r < kFragReads; ++r) {
        __builtin_amdgcn_sched_group_barrier(kMfma, 1, 0);
        __builtin_amdgcn_sched_group_barrier(kDsRd, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(kMfma, kMfmas - kFragReads, 0);
    }
    if (WARM) {
      __builtin_amdgcn_sched_barrier(0);
      if (warm && warm_wave)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, warm_sink, 4, warm_off + uint32_t(kt + kWarmAhead) * warm_kstep, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    frags_mma(f1, acc);
    if (!WARM) __builtin_amdgcn_sched_group_barrier(kMfma, kMfmas, 0);
  };
  // Every call site passes constants, so that each copy of the slice is one scheduling region.
  // Measured: worth 2-4 % per contraction from about 50 slices on, nothing or a small loss at 24.
  constexpr int kWarmMinSlices = 32;
  if (WARM && nk >= kWarmMinSlices) {   // slice kt touches slice kt + 2: all but the last two do
    slice(0, true, true, false);
    for (int kt = 1; kt + kWarmAhead < nk; ++kt) slice(kt, true, true, true);
    slice(nk - 2, true, false, true);
    slice(nk - 1, false, false, false);
  } else {
    for (int kt = 0; kt + 1 < nk; ++kt) slice(kt, true, false, false);
    slice(nk - 1, false, false, false);
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
  if (fast) gemm_tile_dma<true>(operand_row_major(A, lda, M, K), operand_row_major(B, ldb, N, K), K, m0, n0, smem, acc);
  else gemm_tile(A, lda, M, B, ldb, N, K, m0, n0, smem, acc);
}

}  // namespace aero
