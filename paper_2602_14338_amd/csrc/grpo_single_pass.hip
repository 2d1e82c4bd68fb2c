// Forward statistics, clipped loss terms and dlogits of one token row in a single pass over
// HBM (softmax policy of App. C, surrogate of Eq. 2, gradient of App. A.1): the bf16 row is
// read once into registers (19 x 16 bytes per thread at V = 151936 with 1024 threads), the
// log-partition is reduced across the workgroup, and the gradient row is produced from the
// registers - 4 bytes of traffic per logit instead of 6 for a forward pass followed by a
// backward pass.
#include "aero_device.h"

namespace aero {

constexpr int kSpNT = 1024;

// NV vectors of 16 bytes per thread: the first NV - NL live in registers, the last NL in LDS
// (filled directly by buffer_load ... lds, each lane reads back only what its own wave loaded),
// because 20 x 4 data registers plus the working set exceed the 128 VGPRs a 1024-thread
// workgroup may use and the overflow would otherwise go to scratch memory in HBM.
template <int NV, int NL>
__global__ __launch_bounds__(kSpNT) void k_row_single_pass(
    const uint16_t* logits, int64_t T, int V, int64_t ld, const int32_t* __restrict__ targets,
    const float* __restrict__ old_logprob, const int32_t* __restrict__ token_rollout,
    const float* __restrict__ adv, const float* __restrict__ weight, int R, float eps_lo, float eps_hi,
    float grad_scale, int stats_all, float* __restrict__ g_out, float* __restrict__ term_out,
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
  const bool need = signal || (valid && stats_all);   // uniform over the workgroup
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
      if ((i >= R || y >= V) && err_flag) atomicOr(err_flag, i >= R ? AERO_DERR_BAD_ROLLOUT : AERO_DERR_BAD_TARGET);
      g_out[t] = 0.f;
      term_out[t] = 0.f;
      flag_out[t] = 0;
      if (logprob_out) logprob_out[t] = 0.f;
      if (entropy_out) entropy_out[t] = 0.f;
      if (lse_out) lse_out[t] = 0.f;
    }
    zero_fill();
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
  if (tid == 0) {
    g_out[t] = g;
    term_out[t] = term;
    flag_out[t] = flag;
    if (logprob_out) logprob_out[t] = lp;
    if (entropy_out) entropy_out[t] = lse - st.sz / st.s;
    if (lse_out) lse_out[t] = lse;
  }
  if (!drow) return;
  if (g == 0.f) {
    zero_fill();
    return;
  }

  // ---- gradient row from the registers ----
  const float c = -lse * kLog2e;
  const float ng = -g;
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
      for (int e = 0; e < 8; ++e) d[e] = ng * exp2_fast(fmaf(z[e], kLog2e, c));
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
    float d = ng * exp2_fast(fmaf(ztail, kLog2e, c));
    if (jt == y) d += g;
    drow[jt] = f32_to_bf16(d);
  }
}

// True when the single-pass kernel applies: bf16, 16-byte aligned rows, and a row that fits
// the register budget of one 1024-thread workgroup.
bool single_pass_applicable(int32_t dtype, int V, int64_t ld, const void* logits, const void* dlogits) {
  const int nvec = V / 8;
  return dtype == AERO_BF16 && nvec >= kSpNT && nvec <= 20 * kSpNT && (ld % 8) == 0 &&
         reinterpret_cast<uintptr_t>(logits) % 16 == 0 && reinterpret_cast<uintptr_t>(dlogits) % 16 == 0;
}

void single_pass_launch(const void* logits, int64_t T, int V, int64_t ld, const int32_t* targets,
                        const float* old_logprob, const int32_t* token_rollout, const float* adv,
                        const float* weight, int R, float eps_lo, float eps_hi, float grad_scale, int stats_all,
                        float* g, float* term, int32_t* flag, float* logprob_out, float* entropy_out,
                        float* lse_out, void* dlogits, int32_t* err_flag, hipStream_t s) {
  const uint16_t* z = reinterpret_cast<const uint16_t*>(logits);
  uint16_t* dz = reinterpret_cast<uint16_t*>(dlogits);
  if (V / 8 <= 8 * kSpNT)
    hipLaunchKernelGGL((k_row_single_pass<8, 0>), dim3(unsigned(T)), dim3(kSpNT), 0, s, z, T, V, ld, targets, old_logprob,
                       token_rollout, adv, weight, R, eps_lo, eps_hi, grad_scale, stats_all, g, term, flag,
                       logprob_out, entropy_out, lse_out, dz, err_flag);
  else
    hipLaunchKernelGGL((k_row_single_pass<20, 4>), dim3(unsigned(T)), dim3(kSpNT), 4 * kSpNT * 16, s, z, T, V, ld, targets, old_logprob,
                       token_rollout, adv, weight, R, eps_lo, eps_hi, grad_scale, stats_all, g, term, flag,
                       logprob_out, entropy_out, lse_out, dz, err_flag);
}

}  // namespace aero
