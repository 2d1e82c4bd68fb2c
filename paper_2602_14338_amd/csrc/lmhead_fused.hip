// LM head fused into the softmax statistics, the clipped loss and its gradients: logits
// z = hidden @ weight^T exist only as fp32 MFMA accumulator tiles.
//
// Forward   k_compact_valid  rows that have a target are compacted (padding rows take no part in any
//                            contraction; their outputs are written as zeros) and gathered; when a
//                            backward pass follows, the candidates - rows whose rollout has weight and
//                            advantage, i.e. the set AERO's curation leaves - come first
//           k_target_logit   zy = logit of the sampled token (one H-long dot product per row)
//           k_fused_stats    tile of z^T (vocab rows x token columns): every lane owns one token column
//                            per block, so the running (offset, sum exp, sum exp*z) is a per-lane
//                            register recurrence with no shuffles.  On the candidates' token tiles it
//                            also leaves P = exp(z - zy) in bf16 in the K-slab layouts
//                            [vocab/64][token][64] and [vocab chunk][token/64][vocab in chunk][64] that
//                            the two gradient contractions read (2 x T x V x 2 bytes are held)
//           k_fused_combine  merges the per-tile partials of a token -> logprob, entropy, lse
// Backward  token terms + loss reduce (shared with the logits path), then
//           k_candidate_scalars  dz = g (onehot - exp(z - lse)) = scale * P with scale = -g exp(logprob)
//                            per token, except the sampled token's own entry, which is written here; the
//                            scale travels with the other operand (dweight) or is applied after the
//                            contraction (dhidden), so z is never formed a second time
//           k_fused_dz       only when that does not apply (an entropy term in the rows, or a sampled
//                            token more than 40 nats below another logit, where P would leave its safe
//                            range): recompute the z^T tile and store dz itself in the same layouts
//           k_gemm_dh        dhidden partials = (P or dz) @ weight   (split-K over the vocabulary, fp32)
//           k_gemm_dw        dweight = (P or dz)^T @ (scale * hidden)
//           k_scatter_dh     fp32 partials summed in fixed order, times scale -> bf16 dhidden at the original rows
// All contractions use the same 256 x 256 x 64 MFMA tile with both operands K-contiguous.
#include <mutex>

#include "gemm_tile.h"

namespace aero {

aero_status token_terms_from_logprob(int64_t T, int V, const int32_t* targets, const float* logprob,
                                     const float* lse, const float* entropy, const float* old_logprob,
                                     const int32_t* token_rollout, const float* adv, const float* weight, int R,
                                     float eps_lo, float eps_hi, float grad_scale, float ent_coef, float kl_coef,
                                     const float* ref_logprob, float* g, float* term, int32_t* flag, float* ea,
                                     float* eb, float* loss, float* clip_frac, int32_t* err_flag, hipStream_t s);

constexpr size_t kWsAlign = 256;
inline size_t up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ------------------------------------------------------------------------------------------
// workspace
// ------------------------------------------------------------------------------------------
struct FusedPlan {
  int64_t T, T_pad;
  int V, V_ld, H, H_pad, tiles_v, VC, n_chunks;   // VC: vocabulary rows per chunk of the transposed dz
  size_t off_part, off_fidx, off_nf, off_g, off_term, off_flag, off_ea, off_eb, off_ent, off_zy, off_pos, off_nact,
      off_gc, off_lsec, off_yc, off_ac, off_bc, off_scale,
      off_hc, off_hTc, off_WT, off_dz, off_dzT, off_dhacc, total;
};

// dhidden is formed as S split-K partials of the active rows, S chosen on the device so that
// (candidate token tiles) x (H tiles) x S fills the launch grid in whole rounds; the buffer holds S
// stacked copies of the active rows, never more rows than the launch grid covers.  A split's
// operands are addressed with 32-bit byte offsets, so a split may span at most 4 GiB of the dz
// slabs: the grid leaves room for that many splits (plus one) when every token is active.
constexpr int kDhGridMin = 4096;
constexpr int64_t kOperandBytes = int64_t(1) << 32;
static int dh_grid(int64_t T_pad, int H, int V_ld) {
  const int tiles_h = (H + kTile - 1) / kTile;
  const int64_t all = (T_pad / kTile) * tiles_h;
  const int64_t rows = T_pad > int64_t(tiles_h) * kTile ? T_pad : int64_t(tiles_h) * kTile;
  const int64_t s_min = (int64_t(V_ld) * rows * 2 + kOperandBytes - 1) / kOperandBytes;
  const int64_t need = all * (s_min + 1);
  return int(need > kDhGridMin ? need : kDhGridMin);
}
static int64_t dh_part_rows(int64_t T_pad, int H, int V_ld) {
  const int tiles_h = (H + kTile - 1) / kTile;
  const int64_t by_grid = int64_t(dh_grid(T_pad, H, V_ld) / tiles_h + 1) * kTile;   // S x active tiles x H tiles <= grid
  const int64_t by_cap = 64 * T_pad;                                                // S <= 64
  return by_grid < by_cap ? by_grid : by_cap;                                       // >= S * active rows for every S
}

static FusedPlan make_plan(int64_t T, int V, int H) {
  FusedPlan p{};
  p.T = T;
  p.T_pad = int64_t(up(size_t(T > 0 ? T : 1), kTile));
  p.V = V;
  p.V_ld = int(up(size_t(V), kTile));
  p.H = H;
  p.H_pad = int(up(size_t(H), kTile));
  p.tiles_v = p.V_ld / kTile;
  // the transposed dz is stored in vocabulary chunks of at most 2 GiB (T_pad x VC bf16), so that
  // the dweight contraction can address a chunk with 32-bit offsets
  int64_t vc = (int64_t(1024) << 20) / p.T_pad / kTile * kTile;
  if (vc < kTile) vc = kTile;
  if (vc > p.V_ld) vc = p.V_ld;
  p.VC = int(vc);
  p.n_chunks = (p.V_ld + p.VC - 1) / p.VC;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up(bytes, kWsAlign); return at; };
  p.off_part = take(size_t(3) * p.tiles_v * p.T_pad * 4);
  p.off_fidx = take(size_t(p.T_pad) * 4);
  p.off_nf = take(16);
  p.off_g = take(size_t(p.T_pad) * 4);
  p.off_term = take(size_t(p.T_pad) * 4);
  p.off_flag = take(size_t(p.T_pad) * 4);
  p.off_ea = take(size_t(p.T_pad) * 4);
  p.off_eb = take(size_t(p.T_pad) * 4);
  p.off_ent = take(size_t(p.T_pad) * 4);
  p.off_zy = take(size_t(p.T_pad) * 4);
  p.off_pos = take(size_t(p.T_pad) * 4);
  p.off_nact = take(16);
  p.off_gc = take(size_t(p.T_pad) * 4);
  p.off_lsec = take(size_t(p.T_pad) * 4);
  p.off_yc = take(size_t(p.T_pad) * 4);
  p.off_ac = take(size_t(p.T_pad) * 4);
  p.off_bc = take(size_t(p.T_pad) * 4);
  p.off_scale = take(size_t(p.T_pad) * 4);
  p.off_hc = take(size_t(p.T_pad) * H * 2);
  p.off_hTc = take(size_t(p.H_pad) * p.T_pad * 2);
  p.off_WT = take(size_t(p.H_pad) * p.V_ld * 2);
  p.off_dz = take(size_t(p.T_pad) * p.V_ld * 2);
  p.off_dzT = take(size_t(p.n_chunks) * p.VC * p.T_pad * 2);
  p.off_dhacc = take(size_t(dh_part_rows(p.T_pad, H, p.V_ld)) * H * 4);
  p.total = o;
  return p;
}

size_t fused_workspace_bytes(int64_t T, int32_t V, int32_t H) {
  if (T < 0 || V < 1 || H < 1) return 0;
  return make_plan(T, V, H).total;
}

// ------------------------------------------------------------------------------------------
// forward: rows with a target, compacted
// ------------------------------------------------------------------------------------------
// Rows without a target (padding) take no part in the contraction.  Single workgroup, order-preserving
// inside each of two classes: first the candidates - rows that may carry gradient, which is known before the
// forward pass: a target in [0, V), a rollout index in [0, R), weight != 0 and (advantage != 0 or
// every_weighted: an entropy or KL term is on) - then the other rows with a target.
//   fidx[j] = row of position j (-1 past the count), nf = {rows with a target, that rounded up to a tile,
//   candidates, that rounded up to a tile}; pos[t] = position of candidate t, -1 for every other row;
//   nact = {candidates, rounded up, 0}: nact[2] is the flag the forward pass raises when a stored
//   exponential left its safe range (see k_fused_stats).
// token_rollout == null (forward-only call): no candidates, pos / nact are not written.
// Ignored rows get their zero outputs here; a target >= V raises the device error bit.
__global__ __launch_bounds__(1024) void k_compact_valid(
    const int32_t* __restrict__ targets, int64_t T, int64_t T_pad, int V, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R, int every_weighted,
    int32_t* __restrict__ fidx, int32_t* __restrict__ nf, int32_t* __restrict__ pos, int32_t* __restrict__ nact,
    float* __restrict__ logprob, float* __restrict__ entropy, float* __restrict__ lse_out,
    int32_t* __restrict__ err_flag) {
  // each of the 16 waves owns one contiguous range of rows and walks it 64 rows at a time (coalesced
  // reads, ballot + popcount inside the wave): count, exchange the 16 counts, then place
  __shared__ int wsum_c[16], wsum_o[16];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int64_t seg = ((T + 15) / 16 + 63) / 64 * 64;
  const int64_t lo = min(T, wave * seg), hi = min(T, lo + seg);
  const uint64_t below = (uint64_t(1) << lane) - 1;
  // class of row t: 0 = no target, 1 = target only, 2 = candidate
  auto row_class = [&](int64_t t) -> int {
    if (unsigned(targets[t]) >= unsigned(V)) return 0;
    if (!token_rollout) return 1;
    const int i = token_rollout[t];
    if (i < 0 || i >= R) return 1;
    return (weight[i] != 0.f && (every_weighted || adv[i] != 0.f)) ? 2 : 1;
  };
  int cnt_c = 0, cnt_o = 0;
  for (int64_t t0 = lo; t0 < hi; t0 += 64) {
    const int64_t t = t0 + lane;
    const int cls = t < hi ? row_class(t) : 0;
    cnt_c += __popcll(__ballot(cls == 2));
    cnt_o += __popcll(__ballot(cls == 1));
  }
  if (lane == 0) {
    wsum_c[wave] = cnt_c;
    wsum_o[wave] = cnt_o;
  }
  __syncthreads();
  int run_c = 0, run_o = 0, total_c = 0, total_o = 0;
#pragma unroll
  for (int w = 0; w < 16; ++w) {
    run_c += w < wave ? wsum_c[w] : 0;
    run_o += w < wave ? wsum_o[w] : 0;
    total_c += wsum_c[w];
    total_o += wsum_o[w];
  }
  run_o += total_c;   // the other rows follow the candidates
  const int total = total_c + total_o;
  bool bad = false;
  for (int64_t t0 = lo; t0 < hi; t0 += 64) {
    const int64_t t = t0 + lane;
    const bool in = t < hi;
    const int cls = in ? row_class(t) : 0;
    const uint64_t m_c = __ballot(cls == 2), m_o = __ballot(cls == 1);
    int at = -1;
    if (cls == 2) {
      at = run_c + __popcll(m_c & below);
      fidx[at] = int(t);
    } else if (cls == 1) {
      fidx[run_o + __popcll(m_o & below)] = int(t);
    } else if (in) {
      logprob[t] = 0.f;
      lse_out[t] = 0.f;
      if (entropy) entropy[t] = 0.f;
      bad |= targets[t] >= V;
    }
    if (in && pos) pos[t] = at;
    run_c += __popcll(m_c);
    run_o += __popcll(m_o);
  }
  if (bad && err_flag) atomicOr(err_flag, AERO_DERR_BAD_TARGET);
  for (int64_t j = total + tid; j < T_pad; j += 1024) fidx[j] = -1;
  if (tid == 0) {
    nf[0] = total;
    nf[1] = (total + kTile - 1) / kTile * kTile;
    nf[2] = total_c;
    nf[3] = (total_c + kTile - 1) / kTile * kTile;
    if (nact) {
      nact[0] = total_c;
      nact[1] = (total_c + kTile - 1) / kTile * kTile;
      nact[2] = 0;
    }
  }
}

// out[j][:] = in[idx[j]][:] (zeros where idx[j] < 0), H % 8 == 0, 16-byte vectors; one wave per row.
__global__ __launch_bounds__(256) void k_gather_rows(const uint16_t* __restrict__ in, int H,
                                                     const int32_t* __restrict__ idx, int64_t n_rows,
                                                     uint16_t* __restrict__ out) {
  const int lane = threadIdx.x & 63;
  const int64_t j = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (j >= n_rows) return;
  const int src = idx[j];
  for (int k = lane * 8; k < H; k += kWave * 8) {
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (src >= 0) v = *reinterpret_cast<const u32x4_t*>(in + int64_t(src) * H + k);
    *reinterpret_cast<u32x4_t*>(out + j * H + k) = v;
  }
}

// A 256 x 256 bf16 tile (vocabulary rows m0.., token columns n0..) held as packed pairs in the accumulator
// layout, pk[nb][mb][i4] = the four rows acc_row(wm, mb, 4 i4 ..) of column acc_col(wn, nb), leaves in the two
// K-slab layouts the gradient contractions read: [v / 64][token][64] and [v / VC][token / 64][v % VC][64].
// smem: 128 KB, free on entry (every wave past its last read of it).
__device__ __forceinline__ void store_tile_both_layouts(const uint32_t (&pk)[kNB][kMB][4][2], uint16_t* smem, int m0,
                                                        int n0, int64_t T_pad, int VC, uint16_t* __restrict__ dz,
                                                        uint16_t* __restrict__ dzT) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  // The tile leaves through LDS so that both layouts are written with 16-byte coalesced stores.
  // Both LDS images are 256 rows of 512 bytes without padding; a row starts at bank 0, so the
  // positions inside a row are XOR-swizzled with bits of the row index, chosen so that the lanes
  // of every LDS instruction below fall on distinct banks (64 banks of 4 bytes):
  //   image 1, L1[token][vocab]: the 16-byte chunk c = vocab / 8 sits at chunk position
  //     c ^ g(token) (low four bits), g = ((token & 1) << 3) | ((token >> 1) & 7), and the two
  //     8-byte halves of a chunk are exchanged when token & 16.  Writes: 32 lanes = 32 consecutive
  //     tokens, 8 bytes each, one vocabulary position -> 32 distinct bank pairs.  Reads: 16 lanes =
  //     2 tokens x 8 chunks -> the two tokens use different halves of the banks.
  //   image 2, L2[vocab][token]: bits 4-5 of the 4-byte word index are XORed with
  //     s(vocab) = ((vocab & 1) << 1) | ((vocab >> 2) & 1).  Writes: 64 lanes = rows (r, r + 1,
  //     r + 4, r + 5) x 16 consecutive words -> four distinct groups of 16 banks.  Reads: 16 lanes
  //     = 2 rows x 8 chunks, the rows in different halves of the banks.
  auto l1_chunk = [](int tok, int c) -> int {
    const int g = ((tok & 1) << 3) | ((tok >> 1) & 7);
    return (c & ~15) | ((c ^ g) & 15);
  };
  // ---- [token][vocab] ----
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    const int tcol = acc_col(wn, nb, lane);
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int row0 = acc_row(wm, mb, i4 * 4, lane);   // a multiple of 4
        const int half = ((row0 >> 2) ^ (tcol >> 4)) & 1;
        uint2 two = {pk[nb][mb][i4][0], pk[nb][mb][i4][1]};
        *reinterpret_cast<uint2*>(smem + tcol * kTile + l1_chunk(tcol, row0 >> 3) * 8 + half * 4) = two;
      }
  }
  __syncthreads();
  // four 64-wide slabs per tile; consecutive threads walk one slab row by row (8 x 16 bytes per
  // row), so each slab receives one contiguous 32 KB block
#pragma unroll
  for (int k = 0; k < kTile * (kTile / 8) / kGemmNT; ++k) {
    const int u = threadIdx.x + k * kGemmNT;
    const int sl = u >> 11, r = (u >> 3) & 255, c8 = u & 7;
    u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + r * kTile + l1_chunk(r, sl * 8 + c8) * 8);
    if (r & 16) val = u32x4_t{val.z, val.w, val.x, val.y};   // halves were exchanged on the way in
    __builtin_nontemporal_store(val, reinterpret_cast<u32x4_t*>(dz + (int64_t(m0 / 64 + sl) * T_pad + n0 + r) * 64 + c8 * 8));
  }
  __syncthreads();
  // ---- [vocab][token]: neighbouring lanes swap halves so that each writes one (t, t+1) pair ----
  auto l2_word = [](int voc, int w) -> int { return w ^ ((((voc & 1) << 1) | ((voc >> 2) & 1)) << 4); };
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    const int tcol = acc_col(wn, nb, lane);
    const bool odd = lane & 1;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const uint32_t own = pk[nb][mb][i4][h];   // rows r (low half) and r + 1 (high half) at column tcol
          const uint32_t got = __shfl_xor(own, 1, kWave);
          // even lane: row r at columns (tcol, tcol + 1); odd lane: row r + 1 at columns (tcol - 1, tcol)
          const uint32_t outw = odd ? ((got >> 16) | (own & 0xffff0000u)) : ((own & 0xffffu) | (got << 16));
          const int row = acc_row(wm, mb, i4 * 4 + h * 2, lane) + (odd ? 1 : 0);
          *reinterpret_cast<uint32_t*>(smem + row * kTile + l2_word(row, tcol >> 1) * 2) = outw;
        }
  }
  __syncthreads();
  // a tile lies inside one chunk (VC is a multiple of the tile height)
  uint16_t* const dzT_chunk = dzT + int64_t(m0 / VC) * VC * T_pad;
  const int m_in_chunk = m0 % VC;
#pragma unroll
  for (int k = 0; k < kTile * (kTile / 8) / kGemmNT; ++k) {
    const int u = threadIdx.x + k * kGemmNT;
    const int sl = u >> 11, r = (u >> 3) & 255, c8 = u & 7;
    const u32x4_t val = *reinterpret_cast<const u32x4_t*>(smem + r * kTile + l2_word(r, sl * 32 + c8 * 4) * 2);
    __builtin_nontemporal_store(val, reinterpret_cast<u32x4_t*>(dzT_chunk + (int64_t(n0 / 64 + sl) * VC + m_in_chunk + r) * 64 + c8 * 8));
  }
}

// ------------------------------------------------------------------------------------------
// forward: per-tile softmax partials
// ------------------------------------------------------------------------------------------
// grid: xcd_grid(tiles_v * T_pad / 256) workgroups.  Hf holds the compacted rows ([T_pad][H], zero
// past the count); part_* are [tiles_v][T_pad], indexed by compact row.
//
// STORE (a backward pass follows and its rows have the plain form dz = g (onehot - pi)): the token tiles that
// hold candidates also leave P = exp(z - zy) in bf16, zy = the sampled token's own logit (k_target_logit), in
// the two K-slab layouts of the gradient contractions, so that the backward pass need not form z again:
//   dz[t, v] = s_t P[t, v] (v != y_t),  s_t = -g_t exp(logprob_t),  because exp(z - lse) = exp(z - zy) exp(zy - lse);
// the per-token factor s_t moves into the other operand (dweight) or behind the contraction (dhidden), and the
// one entry per row that differs, v = y_t, is overwritten once the log-prob is known (k_candidate_scalars).
// bf16 keeps fp32's exponent range, so P is safe as long as z - zy stays far below 88, and so is the scale
// (about g times the sampled token's probability, which must stay a normal number after it is multiplied
// into a bf16 hidden row) as long as that probability is not below e^-52 or so; a tile that sees
// z - zy > kStoreRange on a candidate column raises nact[2], and the backward pass then forms dz by
// recomputing z as it does for rows with an entropy term (k_fused_dz).  The exponentials are the ones the
// statistics take anyway: P = exp(z - m) * exp(m - zy) with m the running offset of the lane.
constexpr float kStoreRange = 40.f;

// stat_update for 16 values that also hands back the exponentials it formed (relative to st.m on return)
// and the largest of the 16 values.
__device__ __forceinline__ float stat_update_keep(RowStat& st, const float (&z)[16], float (&e)[16]) {
  float vm = z[0];
#pragma unroll
  for (int k = 1; k + 1 < 16; k += 2) vm = max3(vm, z[k], z[k + 1]);
  vm = fmaxf(vm, z[15]);
  const bool grow = vm > st.m + kLazy;
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
    asm volatile("" ::: "memory");
    if (grow) {
      const float f = (st.m == -INFINITY) ? 0.f : exp2_fast((st.m - vm) * kLog2e);
      st.s *= f;
      st.sz *= f;
      st.m = vm;
    }
  }
  const float c = -st.m * kLog2e;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    e[k] = exp2_fast(fmaf(z[k], kLog2e, c));
    st.s += e[k];
    st.sz = fmaf(e[k], z[k], st.sz);
  }
  return vm;
}

template <bool STORE>
__global__ __launch_bounds__(kGemmNT, 2) void k_fused_stats(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Hf, int V, int H, int tiles_v,
    int64_t T_pad, const int32_t* __restrict__ nf, float* __restrict__ part_m,
    float* __restrict__ part_s, float* __restrict__ part_sz, const float* __restrict__ zy, int VC,
    int32_t* __restrict__ nact, uint16_t* __restrict__ dz, uint16_t* __restrict__ dzT) {
  extern __shared__ __align__(16) uint16_t smem[];
  // the tile order covers only the token tiles that hold rows with a target (count known on the
  // device), so that every XCD gets the same number of real tiles; the rest of the grid leaves
  const int tiles_t_act = nf[1] / kTile;
  int tv, tt;
  if (!tile_of_block(tiles_v, tiles_t_act, 0, tiles_v * tiles_t_act, tv, tt)) return;
  const int m0 = tv * kTile, n0 = tt * kTile;
  Acc acc;
  gemm_tile_auto(W, H, V, Hf, H, int(T_pad), H, m0, n0, smem, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const bool full = m0 + kTile <= V;
  const int n_cand = STORE ? nf[2] : 0;
  const bool store = STORE && n0 < n_cand;   // uniform over the workgroup
  uint32_t pk[kNB][kMB][4][2];
  bool wide = false;
  RowStat st[kNB];
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    st[nb] = stat_identity();
    const int col = n0 + acc_col(wn, nb, lane);
    const bool col_cand = store && col < n_cand;
    const float ref = col_cand ? zy[col] : 0.f;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb) {
      if (full) {
        float z[16], e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) z[i] = acc[mb][nb][i];
        if (store) {
          const float vm = stat_update_keep(st[nb], z, e);
          // columns past the candidates keep zeros: their rows of the other operand are zero as well
          const float f = col_cand ? exp2_fast((st[nb].m - ref) * kLog2e) : 0.f;
          wide |= col_cand && vm - ref > kStoreRange;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            pk[nb][mb][i4][0] = pack_bf16x2(e[4 * i4] * f, e[4 * i4 + 1] * f);
            pk[nb][mb][i4][1] = pack_bf16x2(e[4 * i4 + 2] * f, e[4 * i4 + 3] * f);
          }
        } else {
          stat_update<16>(st[nb], z);
        }
      } else {
        float d[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          d[i] = 0.f;
          if (m0 + acc_row(wm, mb, i, lane) < V) {
            const float zi = acc[mb][nb][i];
            float z[1] = {zi};
            stat_update<1>(st[nb], z);
            if (store && col_cand) {
              d[i] = exp2_fast((zi - ref) * kLog2e);
              wide |= zi - ref > kStoreRange;
            }
          }
        }
        if (store) {
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            pk[nb][mb][i4][0] = pack_bf16x2(d[4 * i4], d[4 * i4 + 1]);
            pk[nb][mb][i4][1] = pack_bf16x2(d[4 * i4 + 2], d[4 * i4 + 3]);
          }
        }
      }
    }
    st[nb] = stat_merge(st[nb], stat_shfl_xor(st[nb], 32));   // the two row-halves of the block
  }
  // the two waves that share these token columns (wm = 0, 1) merge through LDS
  RowStat* xch = reinterpret_cast<RowStat*>(smem);   // [256 token columns]
  if (wm == 1 && lane < 32) {
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) xch[wn * 64 + nb * 32 + lane] = st[nb];
  }
  __syncthreads();
  if (wm == 0 && lane < 32) {
#pragma unroll
    for (int nb = 0; nb < kNB; ++nb) {
      const RowStat r = stat_merge(st[nb], xch[wn * 64 + nb * 32 + lane]);
      const int64_t t = n0 + wn * 64 + nb * 32 + lane;   // < T_pad
      const int64_t o = int64_t(tv) * T_pad + t;
      part_m[o] = r.m;
      part_s[o] = r.s;
      part_sz[o] = r.sz;
    }
  }
  if constexpr (STORE) {
    if (store) {
      if (__any(wide) && lane == 0) atomicOr(nact + 2, 1);
      __syncthreads();   // the exchange area is read: LDS is free for the staging of the tile
      store_tile_both_layouts(pk, smem, m0, n0, T_pad, VC, dz, dzT);
    }
  }
}

// zy[j] = logit of the sampled token of compact row j = <hidden row, weight row>, fp32 accumulation of the
// bf16 products in a fixed order; 0 past the count.  One wave per row.
__global__ __launch_bounds__(256) void k_target_logit(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Hf, int H, int64_t T_pad,
    const int32_t* __restrict__ fidx, const int32_t* __restrict__ nf, const int32_t* __restrict__ targets,
    float* __restrict__ zy) {
  const int lane = threadIdx.x & 63;
  const int64_t j = int64_t(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (j >= T_pad) return;
  float dot = 0.f;
  if (j < nf[0]) {   // uniform over the wave
    const int y = targets[fidx[j]];   // 0 <= y < V by construction of fidx
    const uint16_t* hr = Hf + j * H;
    const uint16_t* wr = W + int64_t(y) * H;
    for (int k = lane * 8; k < H; k += kWave * 8) {
      float a[8], b[8];
      unpack8(*reinterpret_cast<const u32x4_t*>(hr + k), a);
      unpack8(*reinterpret_cast<const u32x4_t*>(wr + k), b);
#pragma unroll
      for (int e = 0; e < 8; ++e) dot = fmaf(a[e], b[e], dot);
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off, kWave);
  }
  if (lane == 0) zy[j] = dot;
}

// 64 consecutive compact rows per workgroup of 16 waves.  Phase 1: lane <-> row, the tiles_v
// partials are split over the waves (every load is one coalesced 256-byte row segment) and merged
// through LDS.  Phase 2: each wave takes 4 of the rows, merges their 16 partials and subtracts the
// log-partition from the sampled token's logit (zy, from k_target_logit); results go to the row's
// original position.
constexpr int kCombineTokens = 64;
constexpr int kCombineWaves = 16;
__global__ __launch_bounds__(kCombineWaves * kWave) void k_fused_combine(
    int tiles_v, int64_t T_pad, const int32_t* __restrict__ fidx, const int32_t* __restrict__ nf,
    const float* __restrict__ part_m, const float* __restrict__ part_s, const float* __restrict__ part_sz,
    const float* __restrict__ zy, float* __restrict__ logprob, float* __restrict__ entropy,
    float* __restrict__ lse_out) {
  __shared__ RowStat xs[kCombineWaves][kCombineTokens];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t j0 = int64_t(blockIdx.x) * kCombineTokens;   // j0 + 63 < T_pad
  const int n = nf[0];
  if (j0 >= n) return;
  RowStat st = stat_identity();
  for (int tv = wave; tv < tiles_v; tv += kCombineWaves) {
    const int64_t o = int64_t(tv) * T_pad + j0 + lane;
    st = stat_merge(st, RowStat{part_m[o], part_s[o], part_sz[o]});
  }
  xs[wave][lane] = st;
  __syncthreads();
  constexpr int kPerWave = kCombineTokens / kCombineWaves;
  for (int k4 = 0; k4 < kPerWave; ++k4) {
    const int c = wave * kPerWave + k4;
    const int64_t j = j0 + c;
    if (j >= n) break;   // uniform per wave
    const int64_t t = fidx[j];
    // the 16 wave partials of this row, merged by a 16-lane tree in a fixed order
    RowStat r = lane < kCombineWaves ? xs[lane][c] : stat_identity();
#pragma unroll
    for (int off = kCombineWaves / 2; off > 0; off >>= 1) r = stat_merge(r, stat_shfl_xor(r, off));
    if (lane == 0) {
      const float lse = r.m + logf(r.s);
      logprob[t] = zy[j] - lse;
      lse_out[t] = lse;
      if (entropy) entropy[t] = lse - r.sz / r.s;
    }
  }
}

// ------------------------------------------------------------------------------------------
// backward: compaction, transposes
// ------------------------------------------------------------------------------------------
// Per-candidate scalars, in candidate order (position j <-> token fidx[j]; positions from the count up to
// T_pad are padding without gradient).  The gradient row of a candidate is
//   dz_v = pi_v (ac z_v + bc) + gc 1[v = y],   (ac, bc) = (0, -g) without an entropy term.
// Two ways to get there, chosen here for the whole call (recompute = the caller forces it, or the forward
// pass raised nact[2]):
//   stored       the forward pass left P = exp(z - zy): dz_v = scale P_v with scale = -g exp(logprob), and the
//                entry v = y, g (1 - pi_y) = scale * (-(exp(-logprob) - 1)), is written into both layouts here
//   recompute    k_fused_dz forms dz from gc / lsec / yc / ac / bc; scale = 1
// scale is 0 on padding positions, so that rows the forward tile stored past the candidates drop out.
__global__ __launch_bounds__(256) void k_candidate_scalars(
    const int32_t* __restrict__ fidx, const int32_t* __restrict__ nact, const float* __restrict__ g,
    const float* __restrict__ ea, const float* __restrict__ eb, const float* __restrict__ lse,
    const float* __restrict__ logprob, const int32_t* __restrict__ targets, int64_t T_pad, int VC, int force_recompute,
    float* __restrict__ gc, float* __restrict__ lsec, int32_t* __restrict__ yc, float* __restrict__ ac,
    float* __restrict__ bc, float* __restrict__ scale, uint16_t* __restrict__ dz, uint16_t* __restrict__ dzT) {
  const int64_t j = int64_t(blockIdx.x) * 256 + threadIdx.x;
  if (j >= T_pad) return;
  if (j >= nact[0]) {
    gc[j] = 0.f;
    lsec[j] = 1e30f;   // exp(z - lsec) = 0 whatever z is
    yc[j] = -1;
    ac[j] = 0.f;
    bc[j] = 0.f;
    scale[j] = 0.f;
    return;
  }
  const int64_t t = fidx[j];
  const float gv = g[t];
  const int y = targets[t];
  gc[j] = gv;
  lsec[j] = lse[t];
  yc[j] = y;
  ac[j] = ea ? ea[t] : 0.f;
  bc[j] = ea ? eb[t] : -gv;
  if (force_recompute || nact[2] != 0) {
    scale[j] = 1.f;
    return;
  }
  const float lp = logprob[t];
  scale[j] = -gv * expf(lp);
  const uint16_t own = f32_to_bf16(-expm1f(-lp));
  dz[(int64_t(y / 64) * T_pad + j) * 64 + y % 64] = own;
  dzT[int64_t(y / VC) * VC * T_pad + (int64_t(j / 64) * VC + y % VC) * 64 + j % 64] = own;
}

// Transposes (and optionally gathers) a row-major bf16 matrix into the K-slab layout the GEMM
// tile reads: source row r becomes K index r, source column c becomes operand row c:
//   out[(r / 64) * C_pad * 64 + c * 64 + r % 64] = in[src(r)][c]
// for r < n_k (src = idx[r] if idx else r; src < 0 or src >= rows_in_valid gives 0) and c < C_pad
// (columns c >= C do not exist in `in` and give 0).  Also writes the gathered row-major copy
// gath[r][c] (c < C) when gath != null.  With scale != null the transposed copy holds scale[r] * in[src(r)][c]
// (product in fp32, rounded to bf16 once).  64 x 64 tiles through LDS; grid (n_k / 64, C_pad / 64).
__global__ __launch_bounds__(256) void k_gather_transpose(
    const uint16_t* __restrict__ in, int64_t ld_in, int64_t rows_in_valid, int C, int C_pad,
    const int32_t* __restrict__ idx, int64_t n_k, uint16_t* __restrict__ out, uint16_t* __restrict__ gath,
    int64_t ld_gath, const float* __restrict__ scale) {
  __shared__ uint16_t tile[64][66];
  const int64_t r0 = int64_t(blockIdx.x) * 64;
  const int c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int rr = ty; rr < 64; rr += 4) {
    const int64_t r = r0 + rr;
    const int c = c0 + tx;
    uint16_t v = 0;
    if (r < n_k && c < C) {
      const int64_t src = idx ? int64_t(idx[r]) : r;
      if (src >= 0 && src < rows_in_valid) v = in[src * ld_in + c];
      if (gath) gath[r * ld_gath + c] = v;
      if (scale) v = f32_to_bf16(bf16_to_f32(v) * scale[r]);
    }
    tile[rr][tx] = v;
  }
  __syncthreads();
  // one K-slab holds 64 consecutive r: this block writes rows c0 .. c0+63 of slab blockIdx.x
  uint16_t* slab = out + int64_t(blockIdx.x) * C_pad * 64;
  for (int cc = ty; cc < 64; cc += 4) {
    const int c = c0 + cc;
    if (c < C_pad) slab[int64_t(c) * 64 + tx] = tile[tx][cc];
  }
}

// Same contract, for C % 8 == 0, ld_in % 8 == 0 and 16-byte aligned pointers: every global access
// is a 16-byte vector.  The tile is held in LDS as [r][c] with 32-bit writes; a thread then
// collects 8 consecutive r of one column c for one 16-byte store, threads ordered so that a
// workgroup writes its 64 x 64 block of the slab as one contiguous 8 KB run.
__global__ __launch_bounds__(256) void k_gather_transpose_vec(
    const uint16_t* __restrict__ in, int64_t ld_in, int64_t rows_in_valid, int C, int C_pad,
    const int32_t* __restrict__ idx, int64_t n_k, uint16_t* __restrict__ out, uint16_t* __restrict__ gath,
    int64_t ld_gath, const float* __restrict__ scale) {
  __shared__ uint32_t tile[64][33];   // [r][c / 2]
  const int64_t r0 = int64_t(blockIdx.x) * 64;
  const int c0 = blockIdx.y * 64;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int u = threadIdx.x + k * 256;
    const int rr = u >> 3, c8 = (u & 7) * 8;
    const int64_t r = r0 + rr;
    const int c = c0 + c8;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (r < n_k && c < C) {
      const int64_t src = idx ? int64_t(idx[r]) : r;
      if (src >= 0 && src < rows_in_valid) v = *reinterpret_cast<const u32x4_t*>(in + src * ld_in + c);
      if (gath) *reinterpret_cast<u32x4_t*>(gath + r * ld_gath + c) = v;
      if (scale) {
        const float f = scale[r];
        float x[8];
        unpack8(v, x);
        v.x = pack_bf16x2(x[0] * f, x[1] * f);
        v.y = pack_bf16x2(x[2] * f, x[3] * f);
        v.z = pack_bf16x2(x[4] * f, x[5] * f);
        v.w = pack_bf16x2(x[6] * f, x[7] * f);
      }
    }
    tile[rr][c8 / 2 + 0] = v.x;
    tile[rr][c8 / 2 + 1] = v.y;
    tile[rr][c8 / 2 + 2] = v.z;
    tile[rr][c8 / 2 + 3] = v.w;
  }
  __syncthreads();
  uint16_t* slab = out + int64_t(blockIdx.x) * C_pad * 64;
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int u = threadIdx.x + k * 256;
    const int cc = u >> 3, q = u & 7;   // column cc, K positions 8 q .. 8 q + 7
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t lo = tile[8 * q + 2 * e][cc >> 1], hi = tile[8 * q + 2 * e + 1][cc >> 1];
      w[e] = (cc & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
    }
    const u32x4_t v = {w[0], w[1], w[2], w[3]};
    if (c0 + cc < C_pad) *reinterpret_cast<u32x4_t*>(slab + int64_t(c0 + cc) * 64 + 8 * q) = v;
  }
}

// ------------------------------------------------------------------------------------------
// backward: dz tiles, whole vocabulary
// ------------------------------------------------------------------------------------------
// z^T tile rows = vocab [m0, m0 + 256), columns = compacted tokens.  The bf16 gradient leaves in
// the two K-slab layouts the next two contractions read: dz as [v / 64][token][64] (K = vocab)
// and dzT as [v / VC][token / 64][v % VC][64] (K = tokens, in vocabulary chunks of VC rows so that
// one chunk stays below the 4 GiB a buffer descriptor can address); entries outside the
// vocabulary or the candidate tokens are zero.
// ENT: rows also carry the entropy-bonus term, dz = pi (ac z + bc) + gc onehot; otherwise ac = 0
// and the scale is the per-token constant bc = -g.
// The kernel is the recompute mode of the backward pass (see k_candidate_scalars): with force == 0 it
// leaves at once unless the forward pass raised nact[2].
template <bool ENT>
__global__ __launch_bounds__(kGemmNT, 2) void k_fused_dz(
    const uint16_t* __restrict__ W, const uint16_t* __restrict__ Hc, int V, int H,
    int tiles_v, int64_t T_pad, int VC, int force, const int32_t* __restrict__ nact,
    const float* __restrict__ gc, const float* __restrict__ lsec, const int32_t* __restrict__ yc,
    const float* __restrict__ ac, const float* __restrict__ bc, uint16_t* __restrict__ dz,
    uint16_t* __restrict__ dzT) {
  extern __shared__ __align__(16) uint16_t smem[];
  if (!force && nact[2] == 0) return;   // uniform over the launch
  // tile order over the candidates' token tiles only (see k_fused_stats)
  const int tiles_t_act = nact[1] / kTile;
  int tv, tt;
  if (!tile_of_block(tiles_v, tiles_t_act, 0, tiles_v * tiles_t_act, tv, tt)) return;
  const int m0 = tv * kTile, n0 = tt * kTile;
  Acc acc;
  gemm_tile_auto(W, H, V, Hc, H, int(T_pad), H, m0, n0, smem, acc);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  // dz for this lane's columns, packed to bf16 pairs: pk[nb][mb][i4] = rows row0 .. row0 + 3
  uint32_t pk[kNB][kMB][4][2];
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    const int64_t t = n0 + acc_col(wn, nb, lane);
    const float g = gc[t], ng = bc[t];   // bc = -g without the entropy bonus
    const float a = ENT ? ac[t] : 0.f;
    const float c = -lsec[t] * kLog2e;
    const int yrel = yc[t];        // vocabulary row of the sampled token (-1 on padding columns)
    // Almost every wave holds neither a sampled token's row nor rows past the vocabulary: that
    // case (uniform over the wave) runs without the two per-element tests.
    const bool plain = (m0 + kTile <= V) && !__any(unsigned(yrel - m0 - wm * 128) < 128u);
    if (plain) {
#pragma unroll
      for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          float d[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float z = acc[mb][nb][i4 * 4 + j];
            d[j] = (ENT ? fmaf(a, z, ng) : ng) * exp2_fast(fmaf(z, kLog2e, c));
          }
          pk[nb][mb][i4][0] = pack_bf16x2(d[0], d[1]);
          pk[nb][mb][i4][1] = pack_bf16x2(d[2], d[3]);
        }
    } else {
#pragma unroll
      for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          float d[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int row = m0 + acc_row(wm, mb, i4 * 4 + j, lane);
            const float z = acc[mb][nb][i4 * 4 + j];
            float v = (ENT ? fmaf(a, z, ng) : ng) * exp2_fast(fmaf(z, kLog2e, c));
            if (row == yrel) v += g;
            d[j] = row < V ? v : 0.f;
          }
          pk[nb][mb][i4][0] = pack_bf16x2(d[0], d[1]);
          pk[nb][mb][i4][1] = pack_bf16x2(d[2], d[3]);
        }
    }
  }
  store_tile_both_layouts(pk, smem, m0, n0, T_pad, VC, dz, dzT);
}

// ------------------------------------------------------------------------------------------
// backward: the two gradient GEMMs
// ------------------------------------------------------------------------------------------
// Split-K factor for dhidden, from the number of candidate token tiles (uniform, device side).
// A workgroup's time is its share of the K slices plus a fixed tail (storing its fp32 partial
// tile, worth about 8 slices of main loop); the launch takes ceil(workgroups / 256) such rounds.
// S minimises rounds x (slices / S + 8) among the S whose splits stay addressable: a split's
// slab operands (rows_max rows per 64-wide slice) must span less than 4 GiB.
__device__ __forceinline__ int dh_splits(int active_tiles, int tiles_h, int grid, int slices, int64_t rows_max) {
  const int base = active_tiles * tiles_h;
  if (base == 0) return 0;
  int best = 0;
  int64_t best_cost = INT64_MAX;
  for (int s = 1; base * s <= grid && s <= slices; ++s) {
    const int per = (slices + s - 1) / s;
    if (int64_t(per) * kDK * rows_max * 2 >= (int64_t(1) << 32)) continue;   // not addressable with 32-bit offsets
    const int64_t rounds = (int64_t(base) * s + 255) / 256;
    const int64_t cost = rounds * (per + 8);
    if (cost < best_cost) {
      best_cost = cost;
      best = s;
    }
    if (s >= 64) break;
  }
  return best;
}

// dh_part[s][t][h] = sum_{k in split s} X[t][k] W[k][h], X = the stored exponentials P (or dz itself on the recompute
// route)     M = candidate tokens, N = H, K = vocabulary (padded)
__global__ __launch_bounds__(kGemmNT, 2) void k_gemm_dh(
    const uint16_t* __restrict__ dz, const uint16_t* __restrict__ WT, int H_pad, int vK,
    int H, int tiles_h, int64_t T_pad, const int32_t* __restrict__ nact, float* __restrict__ dh_part) {
  extern __shared__ __align__(16) uint16_t smem[];
  const int n_pad = nact[1];
  const int tiles_t = n_pad / kTile;
  const int nslices = vK / kDK;
  const int S = dh_splits(tiles_t, tiles_h, gridDim.x, nslices, T_pad > H_pad ? T_pad : H_pad);
  const int base = tiles_t * tiles_h;
  const int pid = blockIdx.x;
  if (S == 0 || pid >= base * S) return;   // uniform exit
  // per-XCD contiguous order, split-major: the workgroups resident on one XCD work on the same
  // K range of neighbouring tiles and share their operand slices in that XCD's L2
  const int npid = xcd_regroup(pid, base * S);
  const int split = npid / base;
  int tt, th;
  tile_of_index(npid % base, tiles_t, tiles_h, tt, th);
  const int m0 = tt * kTile, n0 = th * kTile;
  const int per = (nslices + S - 1) / S;
  const int k_begin = min(vK, split * per * kDK);
  const int k_len = max(0, min(vK, (split + 1) * per * kDK) - k_begin);
  Acc acc;
  // both operands are K-slabs over the vocabulary
  gemm_tile_dma<false>(operand_slabs(dz + int64_t(k_begin / kDK) * T_pad * kDK, T_pad, k_len),
                operand_slabs(WT + int64_t(k_begin / kDK) * H_pad * kDK, H_pad, k_len), k_len, m0, n0, smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  float* out = dh_part + int64_t(split) * n_pad * H;
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    const int col = n0 + acc_col(wn, nb, lane);
    if (col >= H) continue;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i)   // written once, read once by the scatter kernel: streamed past the caches
        __builtin_nontemporal_store(acc[mb][nb][i], out + int64_t(m0 + acc_row(wm, mb, i, lane)) * H + col);
  }
}

// dW[m][h] = sum_t XT[m][t] hTc[h][t], hTc = the candidates' hidden rows times their scale     M = V, N = H, K = candidate tokens (padded)
template <bool OUT_BF16>
__global__ __launch_bounds__(kGemmNT, 2) void k_gemm_dw(
    const uint16_t* __restrict__ dzT, const uint16_t* __restrict__ hTc, int VC, int H_pad, int V, int H,
    int tile0, int n_tiles, int tiles_v, int tiles_h, int64_t T_pad, const int32_t* __restrict__ nact,
    int accumulate, void* dW) {
  extern __shared__ __align__(16) uint16_t smem[];
  int tv, th;
  if (!tile_of_block(tiles_v, tiles_h, tile0, n_tiles, tv, th)) return;
  const int m0 = tv * kTile, n0 = th * kTile;
  // the tile's rows lie inside one vocabulary chunk of the transposed dz
  const uint16_t* const dzT_chunk = dzT + int64_t(m0 / VC) * VC * T_pad;
  Acc acc;
  gemm_tile_dma<true>(operand_slabs(dzT_chunk, VC, nact[1]), operand_slabs(hTc, H_pad, nact[1]), nact[1], m0 % VC, n0,
                      smem, acc);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 2, wn = wave & 3;
#pragma unroll
  for (int nb = 0; nb < kNB; ++nb) {
    const int col = n0 + acc_col(wn, nb, lane);
    if (col >= H) continue;
#pragma unroll
    for (int mb = 0; mb < kMB; ++mb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = m0 + acc_row(wm, mb, i, lane);
        if (row < V) {
          const int64_t o = int64_t(row) * H + col;
          // the gradient is not read again by this call: keep it out of the caches.  accumulate (uniform):
          // the tile is added to what the caller's buffer holds (gradient accumulation over micro-batches)
          float v = acc[mb][nb][i];
          if constexpr (OUT_BF16) {
            uint16_t* p = reinterpret_cast<uint16_t*>(dW) + o;
            if (accumulate) v += bf16_to_f32(__builtin_nontemporal_load(p));
            __builtin_nontemporal_store(f32_to_bf16(v), p);
          } else {
            float* p = reinterpret_cast<float*>(dW) + o;
            if (accumulate) v += __builtin_nontemporal_load(p);
            __builtin_nontemporal_store(v, p);
          }
        }
      }
  }
}

// dhidden[t] = bf16(scale[pos[t]] * sum over the split-K partials of row pos[t]) or +0.  One workgroup per
// row; the partials are summed in split order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void k_scatter_dh(const float* __restrict__ dh_part, const int32_t* __restrict__ pos,
                                                    const int32_t* __restrict__ nact, int H, int tiles_h,
                                                    int dh_grid, int slices, int64_t rows_max,
                                                    const float* __restrict__ scale, uint16_t* __restrict__ dhidden) {
  const int64_t t = blockIdx.x;
  const int j = pos[t];
  uint16_t* out = dhidden + t * H;   // H % 8 == 0 and a 16-byte aligned base: rows are whole 16-byte vectors
  const float f = j < 0 ? 0.f : scale[j];
  if (f == 0.f) {   // no gradient row, or one whose token was clipped
    for (int k = threadIdx.x * 8; k < H; k += 256 * 8) *reinterpret_cast<u32x4_t*>(out + k) = u32x4_t{0u, 0u, 0u, 0u};
    return;
  }
  const int n_pad = nact[1];
  const int S = dh_splits(n_pad / kTile, tiles_h, dh_grid, slices, rows_max);   // as the contraction chose it
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  for (int k = threadIdx.x * 4; k < H; k += 256 * 4) {
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
    const float* src = dh_part + int64_t(j) * H + k;
    const int64_t step = int64_t(n_pad) * H;
    int s = 0;
    for (; s + 4 <= S; s += 4) {   // four loads in flight, added in split order
      f32x4_t v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(src + (s + u) * step));
#pragma unroll
      for (int u = 0; u < 4; ++u) acc += v[u];
    }
    for (; s < S; ++s) acc += __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(src + s * step));
    uint2 o;
    o.x = pack_bf16x2(acc.x * f, acc.y * f);
    o.y = pack_bf16x2(acc.z * f, acc.w * f);
    *reinterpret_cast<uint2*>(out + k) = o;
  }
}

// the dz kernel stages a 256 x 256 bf16 tile in LDS after its main loop
static_assert(size_t(kTile) * kTile * 2 <= kWarmSinkOff, "the dz staging tile must end before the warm-up sink");
constexpr size_t kDzLdsBytes = kGemmLdsBytes;

static aero_status set_lds(const void* fn, size_t bytes = kGemmLdsBytes) {
  return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, int(bytes)) == hipSuccess
             ? AERO_OK : AERO_ERR_HIP;
}

}  // namespace aero

extern "C" aero_status aero_lmhead_logprob_fused(
    const void* hidden, const void* weight, int64_t T, int32_t H, int32_t V, const int32_t* targets,
    float* logprob, float* entropy, float* lse, const float* old_logprob, const int32_t* token_rollout,
    const float* adv, const float* weight_rollout, int32_t R, float eps_lo, float eps_hi, float grad_scale,
    float entropy_coef, float kl_coef, const float* ref_logprob, float* loss, float* clip_frac, void* dhidden,
    void* dweight, int32_t dweight_dtype, int32_t* err_flag, void* workspace, size_t workspace_bytes, void* stream) {
  using namespace aero;
  if (!(entropy_coef == entropy_coef) || !(kl_coef == kl_coef)) return AERO_ERR_SHAPE;   // NaN coefficient
  if (old_logprob && kl_coef != 0.f && T > 0 && !ref_logprob) return AERO_ERR_NULL;
  if (T < 0 || T > 0x7fffff00LL || V < 1 || V > (1 << 24) || H < 8 || H % 8 != 0 || H > (1 << 20) || R < 0)
    return AERO_ERR_SHAPE;
  const bool bwd = old_logprob != nullptr;
  const int accumulate = (dweight_dtype & AERO_DW_ACCUMULATE) ? 1 : 0;
  dweight_dtype &= ~AERO_DW_ACCUMULATE;
  if (bwd && dweight_dtype != AERO_F32 && dweight_dtype != AERO_BF16) return AERO_ERR_DTYPE;
  if (!weight) return AERO_ERR_NULL;
  if (T > 0 && (!hidden || !targets || !logprob || !lse)) return AERO_ERR_NULL;
  if (bwd && (!loss || !dweight || (T > 0 && (!token_rollout || !adv || !weight_rollout || !dhidden))))
    return AERO_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(hidden) % 16 || reinterpret_cast<uintptr_t>(weight) % 16) return AERO_ERR_ALIGN;
  if (bwd && reinterpret_cast<uintptr_t>(dhidden) % 16) return AERO_ERR_ALIGN;   // rows are written as 16-byte vectors
  const FusedPlan p = make_plan(T, V, H);
  // operands are addressed with 32-bit byte offsets: every slab operand must stay below 4 GiB
  constexpr size_t kOperandLimit = size_t(1) << 32;
  if (size_t(p.H_pad) * size_t(p.T_pad) * 2 >= kOperandLimit || size_t(p.T_pad) * size_t(p.VC) * 2 >= kOperandLimit ||
      size_t(V) * size_t(H) * 2 >= kOperandLimit)
    return AERO_ERR_SHAPE;
  {  // the split-K dhidden contraction must find a split count whose K ranges stay below that limit
    const int64_t rows = p.T_pad > p.H_pad ? p.T_pad : int64_t(p.H_pad);
    const int64_t s_min = (int64_t(p.V_ld) * rows * 2 + kOperandBytes - 1) / kOperandBytes;
    if (s_min + 1 > 64 || rows * (s_min + 1) >= (int64_t(1) << 25)) return AERO_ERR_SHAPE;
  }
  // one workgroup per 256 x 256 tile: the tile count must fit a launch grid
  if (int64_t(p.tiles_v) * (p.T_pad / kTile) >= (int64_t(1) << 31) - 64) return AERO_ERR_SHAPE;   // grids are rounded up to 64
  if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kWsAlign || workspace_bytes < p.total)
    return AERO_ERR_WORKSPACE;
  hipStream_t s = as_stream(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  const uint16_t* Wp = reinterpret_cast<const uint16_t*>(weight);
  const uint16_t* Hp = reinterpret_cast<const uint16_t*>(hidden);
  float* part_m = reinterpret_cast<float*>(ws + p.off_part);
  float* part_s = part_m + size_t(p.tiles_v) * p.T_pad;
  float* part_sz = part_s + size_t(p.tiles_v) * p.T_pad;
  const int tiles_t = int(p.T_pad / kTile);

  // raising the dynamic-LDS limit is per function; done once per process, safely from any thread
  static std::once_flag attr_once;
  static aero_status attr_rc = AERO_OK;
  std::call_once(attr_once, [] {
    if (set_lds(reinterpret_cast<const void*>(k_fused_stats<false>)) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_fused_stats<true>)) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_fused_dz<false>), kDzLdsBytes) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_fused_dz<true>), kDzLdsBytes) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_gemm_dh)) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_gemm_dw<true>)) != AERO_OK ||
        set_lds(reinterpret_cast<const void*>(k_gemm_dw<false>)) != AERO_OK)
      attr_rc = AERO_ERR_HIP;
  });
  if (attr_rc != AERO_OK) return attr_rc;

  // ---- forward ----
  int32_t* fidx = reinterpret_cast<int32_t*>(ws + p.off_fidx);
  int32_t* nf = reinterpret_cast<int32_t*>(ws + p.off_nf);
  int32_t* pos = reinterpret_cast<int32_t*>(ws + p.off_pos);
  int32_t* nact = reinterpret_cast<int32_t*>(ws + p.off_nact);
  float* zy = reinterpret_cast<float*>(ws + p.off_zy);
  uint16_t* hf = reinterpret_cast<uint16_t*>(ws + p.off_hc);   // rows with a target, candidates first
  uint16_t* dz = reinterpret_cast<uint16_t*>(ws + p.off_dz);
  uint16_t* dzT = reinterpret_cast<uint16_t*>(ws + p.off_dzT);
  const bool ent = bwd && entropy_coef != 0.f;
  // rows with an entropy term are not a multiple of exp(z - zy): their gradient is formed by recomputing z
  const bool stored = bwd && !ent;
  float* ent_arr = entropy ? entropy : (ent ? reinterpret_cast<float*>(ws + p.off_ent) : nullptr);
  if (T > 0) {
    hipLaunchKernelGGL(k_compact_valid, dim3(1), dim3(1024), 0, s, targets, T, p.T_pad, V,
                       bwd ? token_rollout : nullptr, adv, weight_rollout, R, (ent || kl_coef != 0.f) ? 1 : 0, fidx, nf,
                       bwd ? pos : nullptr, bwd ? nact : nullptr, logprob, ent_arr, lse, err_flag);
    hipLaunchKernelGGL(k_gather_rows, dim3(unsigned(p.T_pad / 4)), dim3(256), 0, s, Hp, H, fidx, p.T_pad, hf);
    hipLaunchKernelGGL(k_target_logit, dim3(unsigned(p.T_pad / 4)), dim3(256), 0, s, Wp, hf, H, p.T_pad, fidx, nf,
                       targets, zy);
    {
      const int n = p.tiles_v * tiles_t;
      if (stored)
        hipLaunchKernelGGL(k_fused_stats<true>, dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kGemmLdsBytes, s, Wp, hf,
                           V, H, p.tiles_v, p.T_pad, nf, part_m, part_s, part_sz, zy, p.VC, nact, dz, dzT);
      else
        hipLaunchKernelGGL(k_fused_stats<false>, dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kGemmLdsBytes, s, Wp, hf,
                           V, H, p.tiles_v, p.T_pad, nf, part_m, part_s, part_sz, zy, p.VC, nact, dz, dzT);
    }
    hipLaunchKernelGGL(k_fused_combine, dim3(unsigned(p.T_pad / kCombineTokens)), dim3(kCombineWaves * kWave), 0, s,
                       p.tiles_v, p.T_pad, fidx, nf, part_m, part_s, part_sz, zy, logprob, ent_arr, lse);
  }
  if (!bwd) return launch_status();

  // ---- loss and g_t ----
  float* g = reinterpret_cast<float*>(ws + p.off_g);
  float* term = reinterpret_cast<float*>(ws + p.off_term);
  int32_t* flag = reinterpret_cast<int32_t*>(ws + p.off_flag);
  float* ea = ent ? reinterpret_cast<float*>(ws + p.off_ea) : nullptr;
  float* eb = ent ? reinterpret_cast<float*>(ws + p.off_eb) : nullptr;
  aero_status st = token_terms_from_logprob(T, V, targets, logprob, lse, ent_arr, old_logprob, token_rollout, adv,
                                            weight_rollout, R, eps_lo, eps_hi, grad_scale, entropy_coef, kl_coef,
                                            ref_logprob, g, term, flag, ea, eb, loss, clip_frac, err_flag, s);
  if (st != AERO_OK) return st;

  // ---- per-candidate scalars and operand copies ----
  float* gc = reinterpret_cast<float*>(ws + p.off_gc);
  float* lsec = reinterpret_cast<float*>(ws + p.off_lsec);
  int32_t* yc = reinterpret_cast<int32_t*>(ws + p.off_yc);
  float* ac = reinterpret_cast<float*>(ws + p.off_ac);
  float* bc = reinterpret_cast<float*>(ws + p.off_bc);
  float* scale = reinterpret_cast<float*>(ws + p.off_scale);
  uint16_t* hTc = reinterpret_cast<uint16_t*>(ws + p.off_hTc);
  uint16_t* WT = reinterpret_cast<uint16_t*>(ws + p.off_WT);
  float* dh_acc = reinterpret_cast<float*>(ws + p.off_dhacc);
  const int force = stored ? 0 : 1;
  if (T == 0) {   // no forward kernel ran: an empty candidate set for the kernels below
    hipLaunchKernelGGL(k_compact_valid, dim3(1), dim3(1024), 0, s, targets, T, p.T_pad, V, token_rollout, adv,
                       weight_rollout, R, 0, fidx, nf, pos, nact, logprob, ent_arr, lse, err_flag);
  }
  hipLaunchKernelGGL(k_candidate_scalars, dim3(unsigned(p.T_pad / 256)), dim3(256), 0, s, fidx, nact, g, ea, eb, lse,
                     logprob, targets, p.T_pad, p.VC, force, gc, lsec, yc, ac, bc, scale, dz, dzT);
  const int tiles_h = (H + kTile - 1) / kTile;
  const int grid_dh = dh_grid(p.T_pad, H, p.V_ld);
  const int64_t rows_max = p.T_pad > p.H_pad ? p.T_pad : int64_t(p.H_pad);
  if (T > 0) {   // recompute mode only (the kernel leaves at once otherwise)
    const int n = p.tiles_v * tiles_t;
    if (ent)
      hipLaunchKernelGGL(k_fused_dz<true>, dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kDzLdsBytes, s, Wp, hf, V,
                         H, p.tiles_v, p.T_pad, p.VC, force, nact, gc, lsec, yc, ac, bc, dz, dzT);
    else
      hipLaunchKernelGGL(k_fused_dz<false>, dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kDzLdsBytes, s, Wp, hf, V,
                         H, p.tiles_v, p.T_pad, p.VC, force, nact, gc, lsec, yc, ac, bc, dz, dzT);
  }
  // the candidates' hidden rows, each times its scale, transposed to hTc: K-slabs over the candidate positions
  const bool vec_tr = (H % 8 == 0) && (reinterpret_cast<uintptr_t>(Hp) % 16 == 0) && (reinterpret_cast<uintptr_t>(Wp) % 16 == 0);
  const auto transpose = vec_tr ? k_gather_transpose_vec : k_gather_transpose;
  hipLaunchKernelGGL(transpose, dim3(unsigned(p.T_pad / 64), unsigned(p.H_pad / 64)), dim3(256), 0, s, hf,
                     int64_t(H), p.T_pad, H, p.H_pad, nullptr, p.T_pad, hTc, nullptr, int64_t(0), scale);
  // weight transposed to WT, K-slabs over the vocabulary; rows V..V_ld of the source do not exist -> zeros
  hipLaunchKernelGGL(transpose, dim3(unsigned(p.V_ld / 64), unsigned(p.H_pad / 64)), dim3(256), 0, s, Wp,
                     int64_t(H), int64_t(V), H, p.H_pad, nullptr, int64_t(p.V_ld), WT, nullptr, int64_t(0), nullptr);

  // ---- the two gradient contractions over the whole vocabulary ----
  if (T > 0) {
    // dz columns [V, V_ld) are zero and WT is zero past V: the contraction runs over the padded vocabulary
    hipLaunchKernelGGL(k_gemm_dh, dim3(unsigned(grid_dh)), dim3(kGemmNT), kGemmLdsBytes, s, dz, WT, p.H_pad, p.V_ld, H,
                       tiles_h, p.T_pad, nact, dh_acc);
  }
  // dweight: one launch per chunk of the transposed dz.  VC is sized so that a full chunk is a whole
  // number of rounds of 256 tiles at the two model shapes (measured: 1 % faster than one long launch)
  {
    const int total = p.tiles_v * tiles_h, per = (p.VC / kTile) * tiles_h;
    for (int t0 = 0; t0 < total; t0 += per) {
      const int n = total - t0 < per ? total - t0 : per;
      if (dweight_dtype == AERO_BF16)
        hipLaunchKernelGGL((k_gemm_dw<true>), dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kGemmLdsBytes, s, dzT,
                           hTc, p.VC, p.H_pad, V, H, t0, n, p.tiles_v, tiles_h, p.T_pad, nact, accumulate, dweight);
      else
        hipLaunchKernelGGL((k_gemm_dw<false>), dim3(unsigned(xcd_grid(n))), dim3(kGemmNT), kGemmLdsBytes, s, dzT,
                           hTc, p.VC, p.H_pad, V, H, t0, n, p.tiles_v, tiles_h, p.T_pad, nact, accumulate, dweight);
    }
  }
  if (T > 0)
    hipLaunchKernelGGL(k_scatter_dh, dim3(unsigned(T)), dim3(256), 0, s, dh_acc, pos, nact, H, tiles_h, grid_dh,
                       p.V_ld / kDK, rows_max, scale, reinterpret_cast<uint16_t*>(dhidden));
  return launch_status();
}
