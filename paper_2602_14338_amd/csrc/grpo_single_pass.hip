// Forward statistics, clipped loss terms and dlogits of one token row in a single pass over
// HBM (softmax policy of App. C, surrogate of Eq. 2, gradient of App. A.1): the bf16 row is
// read once into registers (19 x 16 bytes per thread at V = 151936 with 1024 threads), the
// log-partition is reduced across the workgroup, and the gradient row is produced from the
// registers - 4 bytes of traffic per logit instead of 6 for a forward pass followed by a
// backward pass.
#include <mutex>

#include "aero_device.h"

namespace aero {

constexpr int kSpNT = 1024;

// NV vectors of 16 bytes per thread: the first NV - NL live in registers, the last NL in LDS
// (filled directly by buffer_load ... lds, each lane reads back only what its own wave loaded),
// because 20 x 4 data registers plus the working set exceed the 128 VGPRs a 1024-thread
// workgroup may use and the overflow would otherwise go to scratch memory in HBM.
// ENT: the optional terms are on: the entropy bonus (loss and gradient row) and / or the KL penalty
// (a per-token scalar added to the loss term and to g); either coefficient may be 0.
template <int NV, int NL, bool ENT>
__global__ __launch_bounds__(kSpNT) void k_row_single_pass(
    const uint16_t* logits, int64_t T, int V, int64_t ld, const int32_t* __restrict__ targets,
    const float* __restrict__ old_logprob, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R, float eps_lo, float eps_hi,
    float grad_scale, float ent_coef, float kl_coef, const float* __restrict__ ref_logprob, int stats_all,
    float* __restrict__ g_out, float* __restrict__ term_out,
    int32_t* __restrict__ flag_out, float* __restrict__ logprob_out, float* __restrict__ entropy_out,
    float* __restrict__ lse_out, uint16_t* dlogits, int32_t* __restrict__ err_flag) {
  __shared__ RowStat lds[kSpNT / kWave];
  extern __shared__ __align__(16) u32x4_t parked_raw[];   // NL x kSpNT vectors (dynamic LDS)
  u32x4_t(*parked)[kSpNT] = reinterpret_cast<u32x4_t(*)[kSpNT]>(parked_raw);
  constexpr int NR = NV - NL;
  const int64_t t = blockIdx.x;
  const int tid = threadIdx.x;
  const int i = token_rollout[t];
  const int y = targets[t];
  const bool valid = i >= 0 && i < R && y >= 0 && y < V;
  float A = 0.f, w = 0.f;
  if (valid) {
    A = adv[i];
    w = weight[i];
  }
  const bool signal = valid && A != 0.f && w != 0.f;
  const bool bonus = ENT && valid && w != 0.f;          // entropy bonus: every token of a weighted rollout
  const bool need = signal || bonus || (valid && stats_all);   // uniform over the workgroup
  const size_t row_off = size_t(t) * size_t(ld);
  const uint16_t* zrow = logits + row_off;
  uint16_t* drow = dlogits ? dlogits + row_off : nullptr;
  const int nvec = V / 8;
  const u32x4_t zero = {0u, 0u, 0u, 0u};

  auto zero_fill = [&]() {
    if (!drow) return;
    u32x4_t* dv = reinterpret_cast<u32x4_t*>(drow);
    for (int k = tid; k < nvec; k += kSpNT) __builtin_nontemporal_store(zero, dv + k);
    const int j = nvec * 8 + tid;
    if (j < V) drow[j] = 0;
  };

  if (!need) {
    if (tid == 0) {
      // padding / ignored rows (a negative index) are not flagged, whatever their other index holds
      if (i >= 0 && y >= 0 && (i >= R || y >= V) && err_flag)
        atomicOr(err_flag, i >= R ? AERO_DERR_BAD_ROLLOUT : AERO_DERR_BAD_TARGET);
      g_out[t] = 0.f;
      term_out[t] = 0.f;
      flag_out[t] = 0;
      if (logprob_out) logprob_out[t] = 0.f;
      if (entropy_out) entropy_out[t] = 0.f;
      if (lse_out) lse_out[t] = 0.f;
    }
    if (i != AERO_ROW_UNTOUCHED) zero_fill();
    return;
  }

  // ---- the row -> registers.  Buffer loads: one 32-bit offset register instead of a 64-bit
  // pointer per vector, and the descriptor's bounds check returns zeros past the row's end
  // (validity is decided again at use).  aux = 2: non-temporal.
  const __amdgpu_buffer_rsrc_t zsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(zrow), 0, nvec * 16, 0x00020000);
  const uint32_t voff = uint32_t(tid) * 16u;
  u32x4_t v[NR];
#pragma unroll
  for (int u = 0; u < NR; ++u)
    v[u] = __builtin_amdgcn_raw_buffer_load_b128(zsrc, voff + uint32_t(u) * (kSpNT * 16u), 0, 2);
#pragma unroll
  for (int u = NR; u < NV; ++u)   // lane l of wave w lands at parked[u - NR][64 w + l]
    __builtin_amdgcn_raw_ptr_buffer_load_lds(zsrc, &parked[u - NR][(tid >> 6) << 6], 16,
                                             voff + uint32_t(u) * (kSpNT * 16u), 0, 0, 2);
  const int jt = nvec * 8 + tid;   // ragged tail shorter than one vector
  const bool has_tail = jt < V;
  const float ztail = has_tail ? bf16_to_f32(zrow[jt]) : 0.f;
  const float zy = bf16_to_f32(zrow[y]);   // read before any thread may overwrite the row in place

  RowStat st = stat_identity();
#pragma unroll
  for (int u = 0; u < NR; ++u)
  {
    if (tid + u * kSpNT < nvec) {
      float z[8];
      unpack8(v[u], z);
      stat_update<8>(st, z);
    }
    __builtin_amdgcn_sched_barrier(0);   // one vector at a time: keeps temporaries from piling up
  }
  if constexpr (NL > 0) {
    // the compiler does not track loads that land in LDS: wait for this wave's own
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    asm volatile("" ::: "memory");
#pragma unroll
    for (int u = NR; u < NV; ++u) {
      if (tid + u * kSpNT < nvec) {
        const u32x4_t pv = parked[u - NR][tid];
        float z[8];
        unpack8(pv, z);
        stat_update<8>(st, z);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  if (has_tail) {
    float z[1] = {ztail};
    stat_update<1>(st, z);
  }
  st = stat_block_reduce<kSpNT>(st, lds);   // contains the barrier that orders loads before stores
  const float lse = st.m + logf(st.s);
  const float lp = zy - lse;

  // ---- token terms (every thread computes the same scalars) ----
  float g = 0.f, term = 0.f;
  int flag = 0;
  if (signal) {
    const float rho = expf(lp - old_logprob[t]);
    const float lo = 1.f - eps_lo, hi = 1.f + eps_hi;
    const float clipped = fminf(fmaxf(rho, lo), hi);
    const float s = fminf(rho * A, clipped * A);
    const bool unclipped = A > 0.f ? (rho <= hi) : (rho >= lo);
    term = -w * s;
    g = unclipped ? -grad_scale * w * A * rho : 0.f;
    flag = unclipped ? 1 : 2;
  }
  const float ent = lse - st.sz / st.s;
  // gradient row: dz_j = pi_j (a z_j + b) + g 1[j = y]; without the entropy bonus a = 0, b = -g
  if (bonus && kl_coef != 0.f) {   // Eq. 2's beta term: exp(d) - d - 1, d = log pi_ref - log pi
    const float d = ref_logprob[t] - lp;
    const float ed = expf(d);
    term += kl_coef * w * (ed - d - 1.f);
    g += grad_scale * kl_coef * w * (1.f - ed);
  }
  float a = 0.f, ng = -g;
  if (bonus) {
    term -= ent_coef * w * ent;
    a = grad_scale * ent_coef * w;
    ng = a * (ent - lse) - g;
  }
  if (tid == 0) {
    g_out[t] = g;
    term_out[t] = term;
    flag_out[t] = flag;
    if (logprob_out) logprob_out[t] = lp;
    if (entropy_out) entropy_out[t] = ent;
    if (lse_out) lse_out[t] = lse;
  }
  if (!drow) return;
  if (g == 0.f && a == 0.f) {
    zero_fill();
    return;
  }

  // ---- gradient row from the registers ----
  const float c = -lse * kLog2e;
  const __amdgpu_buffer_rsrc_t dsrc = __builtin_amdgcn_make_buffer_rsrc(drow, 0, nvec * 16, 0x00020000);
  // the store offsets are formed again from an opaque copy of the lane offset; otherwise the
  // compiler keeps all NV load offsets alive across the reduction just to reuse them here
  uint32_t voff_st = voff;
  asm volatile("" : "+v"(voff_st));
  const int yvec = y >> 3;
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int k = tid + u * kSpNT;
    if (k < nvec) {
      float z[8], d[8];
      u32x4_t src;
      if constexpr (NL > 0) {
        if (u < NR) src = v[u < NR ? u : 0];
        else src = parked[u >= NR ? u - NR : 0][tid];
      } else {
        src = v[u];
      }
      unpack8(src, z);
#pragma unroll
      for (int e = 0; e < 8; ++e) d[e] = (ENT ? fmaf(a, z[e], ng) : ng) * exp2_fast(fmaf(z[e], kLog2e, c));
      if (k == yvec) {
#pragma unroll
        for (int e = 0; e < 8; ++e) d[e] += (e == (y & 7)) ? g : 0.f;
      }
      u32x4_t o;
      o.x = pack_bf16x2(d[0], d[1]);
      o.y = pack_bf16x2(d[2], d[3]);
      o.z = pack_bf16x2(d[4], d[5]);
      o.w = pack_bf16x2(d[6], d[7]);
      __builtin_amdgcn_raw_buffer_store_b128(o, dsrc, voff_st + uint32_t(u) * (kSpNT * 16u), 0, 2);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (has_tail) {
    float d = (ENT ? fmaf(a, ztail, ng) : ng) * exp2_fast(fmaf(ztail, kLog2e, c));
    if (jt == y) d += g;
    drow[jt] = f32_to_bf16(d);
  }
}

// ------------------------------------------------------------------------------------------
// Streaming variant for long rows.  One persistent 1024-thread workgroup per CU walks rows
// t = blockIdx.x, + gridDim.x, ...  The first NL vectors of every thread live in LDS, filled by
// buffer_load ... lds into wave-private slots; as soon as a slot has been turned into gradient
// and stored, the same slot is refilled with the NEXT row's vector, so the CU keeps reads in
// flight during its store phase (a workgroup of this size cannot share a CU with a second one).
// The remaining NV - NL vectors are ordinary register loads issued at the top of a row.
// Rows are handed out through a global counter (padding and zero-advantage rows cost far less
// than gradient rows, a fixed stride would leave CUs idle); a workgroup always knows its next
// row one row ahead, and leaves when the counter has passed T.  The counter indexes a row order
// in which the rows that are read come first and the rows that are only zero-filled last
// (k_row_order): the memory system then sees a read+write phase followed by a write-only
// phase instead of a mix of the two, which is worth several percent on padded batches.
// Rows marked AERO_ROW_UNTOUCHED are in neither part: their gradient row is not written, their
// scalars are zeroed by k_row_order, and this kernel never sees them.
// ------------------------------------------------------------------------------------------
struct RowInfo {
  int y;
  float A, w;
  bool valid, signal, bonus, need;
};

// every_weighted: the entropy bonus is on, rows of weighted rollouts with advantage 0 count too
__device__ __forceinline__ RowInfo row_info(int64_t t, int64_t T, int V, int R, const int32_t* targets,
                                            const int32_t* token_rollout, const float* adv, const float* weight,
                                            int stats_all, bool every_weighted) {
  RowInfo r{0, 0.f, 0.f, false, false, false, false};
  if (t >= T) return r;
  const int i = token_rollout[t];
  r.y = targets[t];
  r.valid = i >= 0 && i < R && r.y >= 0 && r.y < V;
  if (r.valid) {
    r.A = adv[i];
    r.w = weight[i];
  }
  r.signal = r.valid && r.A != 0.f && r.w != 0.f;
  r.bonus = every_weighted && r.valid && r.w != 0.f;
  r.need = r.signal || r.bonus || (r.valid && stats_all);
  return r;
}

// order[0 .. n) = rows with need, order[T - m .. T) = the m rows that are only zero-filled, each part in
// no particular order (wave-sized runs are placed by two atomic counters: ctr[1] from the front, ctr[2]
// from the back).  The u rows marked AERO_ROW_UNTOUCHED are placed nowhere (n + m + u = T, the gap in the
// middle has u entries; ctr[3] counts them) and get their per-row scalars, all zero, here.
__global__ __launch_bounds__(256) void k_row_order(int64_t T, int V, int R, const int32_t* __restrict__ targets,
                                                   const int32_t* __restrict__ token_rollout,
                                                   const float* __restrict__ adv, const float* __restrict__ weight,
                                                   int stats_all, int every_weighted, int32_t* __restrict__ ctr,
                                                   int32_t* __restrict__ order, float* __restrict__ g_out,
                                                   float* __restrict__ term_out, int32_t* __restrict__ flag_out,
                                                   float* __restrict__ logprob_out, float* __restrict__ entropy_out,
                                                   float* __restrict__ lse_out) {
  const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int lane = threadIdx.x & 63;
  const bool in = t < T;
  const bool untouched = in && token_rollout[t] == AERO_ROW_UNTOUCHED;
  const bool need = row_info(t, T, V, R, targets, token_rollout, adv, weight, stats_all, every_weighted != 0).need;
  const uint64_t m_need = __ballot(in && need), m_rest = __ballot(in && !need && !untouched);
  const uint64_t m_unt = __ballot(untouched);
  const uint64_t below = (uint64_t(1) << lane) - 1;
  int base_need = 0, base_rest = 0;
  if (lane == 0) {
    if (m_need) base_need = atomicAdd(ctr + 1, __popcll(m_need));
    if (m_rest) base_rest = atomicAdd(ctr + 2, __popcll(m_rest));
    if (m_unt) atomicAdd(ctr + 3, __popcll(m_unt));
  }
  if (untouched) {
    g_out[t] = 0.f;
    term_out[t] = 0.f;
    flag_out[t] = 0;
    if (logprob_out) logprob_out[t] = 0.f;
    if (entropy_out) entropy_out[t] = 0.f;
    if (lse_out) lse_out[t] = 0.f;
  }
  base_need = __shfl(base_need, 0, kWave);
  base_rest = __shfl(base_rest, 0, kWave);
  if (in && need) order[base_need + __popcll(m_need & below)] = int32_t(t);
  if (in && !need && !untouched) order[T - 1 - (base_rest + __popcll(m_rest & below))] = int32_t(t);
}

template <int NV, int NL, bool ENT>
__global__ __launch_bounds__(kSpNT) void k_row_stream(
    const uint16_t* logits, int64_t T, int V, int64_t ld, const int32_t* __restrict__ targets,
    const float* __restrict__ old_logprob, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R, float eps_lo, float eps_hi,
    float grad_scale, float ent_coef, float kl_coef, const float* __restrict__ ref_logprob, int stats_all,
    float* __restrict__ g_out, float* __restrict__ term_out,
    int32_t* __restrict__ flag_out, float* __restrict__ logprob_out, float* __restrict__ entropy_out,
    float* __restrict__ lse_out, uint16_t* dlogits, int32_t* __restrict__ err_flag, int32_t* row_counter,
    const int32_t* __restrict__ order) {
  // positions 0 .. P of the hand-out skip the gap that the untouched rows leave in the row order
  const int n_front = row_counter[1];
  const int n_gap = row_counter[3];
  const int64_t P = T - n_gap;
  auto row_at = [&](int64_t p) -> int64_t { return p < P ? order[p < n_front ? p : p + n_gap] : T; };
  __shared__ RowStat lds[2][kSpNT / kWave];   // alternating: one barrier per row is enough
  __shared__ int s_next;
  extern __shared__ __align__(16) u32x4_t slots_raw[];   // NL x kSpNT vectors
  u32x4_t(*slots)[kSpNT] = reinterpret_cast<u32x4_t(*)[kSpNT]>(slots_raw);
  constexpr int NR = NV - NL;
  const int tid = threadIdx.x;
  const int nvec = V / 8;
  const uint32_t voff = uint32_t(tid) * 16u;
  const u32x4_t zero = {0u, 0u, 0u, 0u};
  const int jt = nvec * 8 + tid;   // ragged tail shorter than one vector
  const bool has_tail = jt < V;

  auto row_rsrc = [&](const uint16_t* base, int64_t row) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base + size_t(row) * size_t(ld)), 0, nvec * 16,
                                             0x00020000);
  };
  auto dma_slot = [&](__amdgpu_buffer_rsrc_t src, int u) {   // lane l of wave w lands at slots[u][64 w + l]
    __builtin_amdgcn_raw_ptr_buffer_load_lds(src, &slots[u][(tid >> 6) << 6], 16,
                                             voff + uint32_t(u) * (kSpNT * 16u), 0, 0, 2);
  };

  // the first gridDim.x positions of the row order are assigned by workgroup id; the counter
  // starts at gridDim.x.  pn = position of the next row, tn = that row (T = none left)
  int64_t t = row_at(blockIdx.x);
  if (tid == 0) s_next = atomicAdd(row_counter, 1);
  __syncthreads();
  int64_t pn = s_next;
  int64_t tn = row_at(pn);
  RowInfo cur = row_info(t, T, V, R, targets, token_rollout, adv, weight, stats_all, ENT);
  if (cur.need) {
    const __amdgpu_buffer_rsrc_t src = row_rsrc(logits, t);
#pragma unroll
    for (int u = 0; u < NL; ++u) dma_slot(src, u);
  }

  int reduces = 0;   // selects the LDS buffer of the next reduction
  while (t < T) {
    const RowInfo nxt = row_info(tn, T, V, R, targets, token_rollout, adv, weight, stats_all, ENT);
    const uint16_t* zrow = logits + size_t(t) * size_t(ld);
    uint16_t* drow = dlogits ? dlogits + size_t(t) * size_t(ld) : nullptr;
    const __amdgpu_buffer_rsrc_t nsrc = row_rsrc(logits, nxt.need ? tn : t);
    float g = 0.f, term = 0.f, lp = 0.f, ent = 0.f, lse = 0.f;
    float ea = 0.f;   // entropy bonus: grad_scale c w of this row (ENT only)
    int flag = 0;
    u32x4_t v[NR];
    float ztail = 0.f;

    if (cur.need) {   // uniform over the workgroup
      const __amdgpu_buffer_rsrc_t zsrc = row_rsrc(logits, t);
#pragma unroll
      for (int u = 0; u < NR; ++u)
        v[u] = __builtin_amdgcn_raw_buffer_load_b128(zsrc, voff + uint32_t(NL + u) * (kSpNT * 16u), 0, 2);
      ztail = has_tail ? bf16_to_f32(zrow[jt]) : 0.f;
      const float zy = bf16_to_f32(zrow[cur.y]);   // read before any thread may overwrite the row in place
      // Loads return in order and at least NR + 1 of them were issued just above: once no more
      // than NR memory operations are outstanding, the older loads into this wave's LDS slots
      // have landed (the compiler does not track those; stores may retire in any order, they
      // only make the wait longer).
      static_assert(NR <= 15, "immediate below holds vmcnt in 4 bits");
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_waitcnt(0x0F70 | NR);
      asm volatile("" ::: "memory");
      RowStat st = stat_identity();
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        if (tid + u * kSpNT < nvec) {
          const u32x4_t pv = slots[u][tid];
          float z[8];
          unpack8(pv, z);
          stat_update<8>(st, z);
        }
        __builtin_amdgcn_sched_barrier(0);   // one vector at a time: keeps temporaries from piling up
      }
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        if (tid + (NL + u) * kSpNT < nvec) {
          float z[8];
          unpack8(v[u], z);
          stat_update<8>(st, z);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (has_tail) {
        float z[1] = {ztail};
        stat_update<1>(st, z);
      }
      st = stat_block_reduce<kSpNT>(st, lds[reduces++ & 1]);   // its barrier also orders loads before stores
      lse = st.m + logf(st.s);
      lp = zy - lse;
      ent = lse - st.sz / st.s;
      if (cur.signal) {   // every thread computes the same scalars
        const float rho = expf(lp - old_logprob[t]);
        const float lo = 1.f - eps_lo, hi = 1.f + eps_hi;
        const float clipped = fminf(fmaxf(rho, lo), hi);
        const float s = fminf(rho * cur.A, clipped * cur.A);
        const bool unclipped = cur.A > 0.f ? (rho <= hi) : (rho >= lo);
        term = -cur.w * s;
        g = unclipped ? -grad_scale * cur.w * cur.A * rho : 0.f;
        flag = unclipped ? 1 : 2;
      }
      if constexpr (ENT) {
        if (cur.bonus) {
          if (kl_coef != 0.f) {   // Eq. 2's beta term: exp(d) - d - 1, d = log pi_ref - log pi
            const float d = ref_logprob[t] - lp;
            const float ed = expf(d);
            term += kl_coef * cur.w * (ed - d - 1.f);
            g += grad_scale * kl_coef * cur.w * (1.f - ed);
          }
          term -= ent_coef * cur.w * ent;
          ea = grad_scale * ent_coef * cur.w;
        }
      }
    }
    if (tid == 0) {
      if (!cur.valid && err_flag) {
        const int i = token_rollout[t];
        if (i >= 0 && cur.y >= 0 && (i >= R || cur.y >= V))   // padding / ignored rows are not flagged
          atomicOr(err_flag, i >= R ? AERO_DERR_BAD_ROLLOUT : AERO_DERR_BAD_TARGET);
      }
      g_out[t] = g;
      term_out[t] = term;
      flag_out[t] = flag;
      if (logprob_out) logprob_out[t] = lp;
      if (entropy_out) entropy_out[t] = ent;
      if (lse_out) lse_out[t] = lse;
    }

    if (drow && (g != 0.f || (ENT && ea != 0.f))) {
      const float c = -lse * kLog2e;
      // gradient row: dz_j = pi_j (a z_j + ng) + g 1[j = y]; without the entropy bonus a = 0, ng = -g
      const float a = ea;
      const float ng = ENT ? ea * (ent - lse) - g : -g;
      const __amdgpu_buffer_rsrc_t dsrc = row_rsrc(dlogits, t);
      uint32_t voff_st = voff;   // opaque copy: keeps the load offsets from being kept alive for reuse
      asm volatile("" : "+v"(voff_st));
      const int y = cur.y, yvec = y >> 3;
      auto grad_vec = [&](const u32x4_t& src, int k) -> u32x4_t {
        float z[8], d[8];
        unpack8(src, z);
#pragma unroll
        for (int e = 0; e < 8; ++e) d[e] = (ENT ? fmaf(a, z[e], ng) : ng) * exp2_fast(fmaf(z[e], kLog2e, c));
        if (k == yvec) {
#pragma unroll
          for (int e = 0; e < 8; ++e) d[e] += (e == (y & 7)) ? g : 0.f;
        }
        u32x4_t o;
        o.x = pack_bf16x2(d[0], d[1]);
        o.y = pack_bf16x2(d[2], d[3]);
        o.z = pack_bf16x2(d[4], d[5]);
        o.w = pack_bf16x2(d[6], d[7]);
        return o;
      };
#pragma unroll
      for (int u = 0; u < NL; ++u) {   // LDS part first: each slot is refilled right after its last use
        const int k = tid + u * kSpNT;
        const u32x4_t pv = slots[u][tid];
        if (k < nvec) __builtin_amdgcn_raw_buffer_store_b128(grad_vec(pv, k), dsrc, voff_st + uint32_t(u) * (kSpNT * 16u), 0, 2);
        asm volatile("" ::: "memory");
        if (nxt.need) dma_slot(nsrc, u);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int u = 0; u < NR; ++u) {
        const int k = tid + (NL + u) * kSpNT;
        if (k < nvec) __builtin_amdgcn_raw_buffer_store_b128(grad_vec(v[u], k), dsrc, voff_st + uint32_t(NL + u) * (kSpNT * 16u), 0, 2);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (has_tail) {
        float d = (ENT ? fmaf(a, ztail, ng) : ng) * exp2_fast(fmaf(ztail, kLog2e, c));
        if (jt == y) d += g;
        drow[jt] = f32_to_bf16(d);
      }
    } else {
      // this row's slots are no longer needed: make sure every read of them has returned
      __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0)
      asm volatile("" ::: "memory");
      if (nxt.need) {
#pragma unroll
        for (int u = 0; u < NL; ++u) dma_slot(nsrc, u);
      }
      if (drow) {   // zero fill
        u32x4_t* dv = reinterpret_cast<u32x4_t*>(drow);
        for (int k = tid; k < nvec; k += kSpNT) __builtin_nontemporal_store(zero, dv + k);
        if (has_tail) drow[jt] = 0;
      }
    }
    // hand-over: the row after the next one is drawn now (all threads have read s_next)
    __syncthreads();
    if (tid == 0) s_next = pn < P ? atomicAdd(row_counter, 1) : int(T);
    __syncthreads();
    cur = nxt;
    t = tn;
    pn = s_next;
    tn = row_at(pn);
  }
}

// ctr[0]: row counter of k_row_stream (starts past the rows assigned by workgroup id),
// ctr[1], ctr[2]: fill counters of k_row_order, ctr[3]: its count of untouched rows
__global__ void k_set_counter(int32_t* ctr, int32_t v) {
  ctr[0] = v;
  ctr[1] = 0;
  ctr[2] = 0;
  ctr[3] = 0;
}

// True when the single-pass kernel applies: bf16, 16-byte aligned rows, and a row that fits
// the register budget of one 1024-thread workgroup.
bool single_pass_applicable(int32_t dtype, int V, int64_t ld, const void* logits, const void* dlogits) {
  const int nvec = V / 8;
  return dtype == AERO_BF16 && nvec >= kSpNT && nvec <= 20 * kSpNT && (ld % 8) == 0 &&
         reinterpret_cast<uintptr_t>(logits) % 16 == 0 && reinterpret_cast<uintptr_t>(dlogits) % 16 == 0;
}

template <bool ENT>
static aero_status single_pass_launch_t(const uint16_t* z, int64_t T, int V, int64_t ld, const int32_t* targets,
                                        const float* old_logprob, const int32_t* token_rollout, const float* adv,
                                        const float* weight, int R, float eps_lo, float eps_hi, float grad_scale,
                                        float ent_coef, float kl_coef, const float* ref_logprob, int stats_all,
                                        float* g, float* term, int32_t* flag,
                                        float* logprob_out, float* entropy_out, float* lse_out, uint16_t* dz,
                                        int32_t* err_flag, int32_t* row_counter, int32_t* row_order, hipStream_t s) {
  if (V / 8 <= 8 * kSpNT) {
    hipLaunchKernelGGL((k_row_single_pass<8, 0, ENT>), dim3(unsigned(T)), dim3(kSpNT), 0, s, z, T, V, ld, targets,
                       old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi, grad_scale, ent_coef, kl_coef, ref_logprob,
                       stats_all, g, term, flag, logprob_out, entropy_out, lse_out, dz, err_flag);
    return AERO_OK;
  }
  constexpr int NL = 9;
  constexpr int kLdsBytes = NL * kSpNT * 16;   // 144 KB of wave-private slots
  // raising the dynamic-LDS limit is per function; done once per process, safely from any thread
  static std::once_flag attr_once;
  static hipError_t attr_rc = hipSuccess;
  std::call_once(attr_once, [] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(k_row_stream<20, NL, ENT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  });
  if (attr_rc != hipSuccess) return AERO_ERR_HIP;
  int dev = 0, cus = 256;
  if (hipGetDevice(&dev) == hipSuccess) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cus = n;
  }
  const unsigned grid = unsigned(T < cus ? T : cus);   // one persistent workgroup per CU
  hipLaunchKernelGGL(k_set_counter, dim3(1), dim3(1), 0, s, row_counter, int32_t(grid));
  hipLaunchKernelGGL(k_row_order, dim3(unsigned((T + 255) / 256)), dim3(256), 0, s, T, V, R, targets, token_rollout,
                     adv, weight, stats_all, ENT ? 1 : 0, row_counter, row_order, g, term, flag, logprob_out,
                     entropy_out, lse_out);
  hipLaunchKernelGGL((k_row_stream<20, NL, ENT>), dim3(grid), dim3(kSpNT), kLdsBytes, s, z, T, V, ld, targets,
                     old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi, grad_scale, ent_coef, kl_coef, ref_logprob,
                     stats_all, g, term, flag, logprob_out, entropy_out, lse_out, dz, err_flag, row_counter, row_order);
  return AERO_OK;
}

// A non-zero entropy or KL coefficient selects the kernels that carry the optional terms.
aero_status single_pass_launch(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                               const float* old_logprob, const int32_t* token_rollout, const float* adv,
                               const float* weight, int R, float eps_lo, float eps_hi, float grad_scale,
                               float ent_coef, float kl_coef, const float* ref_logprob, int stats_all, float* g,
                               float* term, int32_t* flag, float* logprob_out, float* entropy_out, float* lse_out,
                               void* dlogits, int32_t* err_flag, int32_t* row_counter, int32_t* row_order,
                               hipStream_t s) {
  const uint16_t* z = reinterpret_cast<const uint16_t*>(logits);
  uint16_t* dz = reinterpret_cast<uint16_t*>(dlogits);
  if (ent_coef != 0.f || kl_coef != 0.f)
    return single_pass_launch_t<true>(z, T, V, ld, targets, old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi,
                                      grad_scale, ent_coef, kl_coef, ref_logprob, stats_all, g, term, flag, logprob_out,
                                      entropy_out, lse_out, dz, err_flag, row_counter, row_order, s);
  return single_pass_launch_t<false>(z, T, V, ld, targets, old_logprob, token_rollout, adv, weight, R, eps_lo, eps_hi,
                                     grad_scale, 0.f, 0.f, nullptr, stats_all, g, term, flag, logprob_out, entropy_out,
                                     lse_out, dz, err_flag, row_counter, row_order, s);
}

}  // namespace aero
