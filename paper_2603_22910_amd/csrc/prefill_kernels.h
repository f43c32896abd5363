// Causal prefill attention (Eq. 7 with a causal mask) on bf16 MFMA, over the
// target layer's retained heads (read from the cache) and its predicted heads
// (read from the workspace where the predictor product put them once for the
// whole chunk).
//
// One workgroup = 128 consecutive queries of one query head; each of its four
// waves owns 32 queries.  Per 64-key tile a wave computes
//   S^T = K Q^T   (rows = keys, lanes = queries)  -> the softmax of a query is
//                  a reduction over the lane's own registers plus its partner
//                  lane (lane ^ 32), and
//   O^T += V^T P^T (rows = head dims, lanes = queries) -> the running rescale
//                  of O is lane-local too, and P^T is used straight from the
//                  S^T accumulators (rounded to bf16): it never goes to LDS.
// The key index a (lane half, element) slot of the MFMA k-dimension stands for
// is free as long as both operands agree; V^T fragments are read from LDS in
// the order the S^T accumulator layout dictates.
#pragma once
#include "common.h"
#include "fused_decode.h"

namespace echokv {
namespace prefill {

constexpr int BQ = 128, BKV = 64, NTHREADS = 256;

struct Args {
  const bf16_t* k_ret; const bf16_t* v_ret;   // retained heads, first row of the sequence, stride m
  const bf16_t* k_hat; const bf16_t* v_hat;   // predicted heads, row 0 = token 0, stride d_out
  const bf16_t* q;                            // [T_q, H_q, d]
  void* out; float* lse;                      // [T_q, H_q, d], [T_q, H_q]
  int32_t H_q, G, m, d_out, n_ret_heads, T_q, q_pos0, out_bf16;
  float scale;
};

template <int HD> struct Cfg {
  static constexpr int CH = HD / 8;             // 16-byte chunks per K row
  static constexpr int KSTEPS = HD / 16;        // MFMA k-steps over the head dim
  static constexpr int CB = HD / 32;            // 32-row blocks of O^T
  static constexpr int KTILE_BYTES = BKV * HD * 2;
  static constexpr int VTILE_BYTES = HD * BKV * 2;
  __device__ static __forceinline__ int kswz(int r) {
    return CH == 16 ? (r & 15) : ((r ^ (r >> 3)) & 7);
  }
};
__device__ __forceinline__ int vswz(int r) { return (r ^ (r >> 3)) & 7; }

template <int HD>
__global__ __launch_bounds__(NTHREADS, 2) void prefill_attn_kernel(Args a) {
  using C = Cfg<HD>;
  __shared__ __attribute__((aligned(16))) char sk[2][C::KTILE_BYTES];
  __shared__ __attribute__((aligned(16))) char sv[2][C::VTILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int h = blockIdx.y;
  const int nqb = (a.T_q + BQ - 1) / BQ;
  const int qb = nqb - 1 - blockIdx.x;            // longest (latest) query blocks first
  const int i0 = qb * BQ;
  const int Ltot = a.q_pos0 + a.T_q;
  const int kvh = h / a.G;
  const bf16_t* kbase; const bf16_t* vbase; int64_t ld;
  if (kvh < a.n_ret_heads) { kbase = a.k_ret + kvh * HD; vbase = a.v_ret + kvh * HD; ld = a.m; }
  else { const int c = (kvh - a.n_ret_heads) * HD; kbase = a.k_hat + c; vbase = a.v_hat + c; ld = a.d_out; }

  // this lane's query (clamped; clamped duplicates are not written back)
  const int qi = i0 + wave * 32 + lr;
  const int qic = min(qi, a.T_q - 1);
  const int qpos = a.q_pos0 + qic;
  bf16x8_t qf[C::KSTEPS];
  {
    const bf16_t* qp = a.q + ((int64_t)qic * a.H_q + h) * HD + lh * 8;
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) qf[kk] = *reinterpret_cast<const bf16x8_t*>(qp + kk * 16);
  }
  floatx16_t oacc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float scale2 = a.scale * 1.44269504088896340736f;    // softmax in base 2: exp(x) = 2^(x log2 e)
  // smallest query position among this wave's lanes (lane 0 of either half)
  const int qpos_min = a.q_pos0 + min(i0 + wave * 32, a.T_q - 1);

  const int kv_end = min(Ltot, a.q_pos0 + min(i0 + BQ, a.T_q));   // keys any query of the block sees
  const int ntiles = (kv_end + BKV - 1) / BKV;

  // staging: K tile = BKV*CH chunks over 256 threads; V tile = (BKV/8)*(HD/8) 8x8 blocks
  constexpr int KLD = BKV * C::CH / NTHREADS;      // 4 (HD=128) or 2 (HD=64)
  constexpr int VBLK = (BKV / 8) * (HD / 8);       // 128 or 64 blocks
  fused::u32x4_t kst[KLD], vst[8];
  const int v_cb = tid % (HD / 8), v_kb = tid / (HD / 8);     // V block of this thread (tid < VBLK)

  auto fetch = [&](int t) {
    const int kv0 = t * BKV;
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int idx = i * NTHREADS + tid, row = idx / C::CH, c = idx % C::CH;
      const int key = min(kv0 + row, Ltot - 1);
      kst[i] = *reinterpret_cast<const fused::u32x4_t*>(kbase + (int64_t)key * ld + c * 8);
    }
    if (tid < VBLK) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int key = min(kv0 + v_kb * 8 + i, Ltot - 1);
        vst[i] = *reinterpret_cast<const fused::u32x4_t*>(vbase + (int64_t)key * ld + v_cb * 8);
      }
    }
  };
  auto stash = [&](int stage) {
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int idx = i * NTHREADS + tid, row = idx / C::CH, c = idx % C::CH;
      *reinterpret_cast<fused::u32x4_t*>(sk[stage] + (row * C::CH + (c ^ C::kswz(row))) * 16) = kst[i];
    }
    if (tid < VBLK) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {      // V^T row c = 8 v_cb + j gets keys 8 v_kb .. +7
        fused::u32x4_t o;
#pragma unroll
        for (int pq = 0; pq < 4; ++pq)
          o[pq] = __builtin_amdgcn_perm(vst[2 * pq + 1][j >> 1], vst[2 * pq][j >> 1],
                                        (j & 1) ? 0x07060302u : 0x05040100u);
        const int c = v_cb * 8 + j;
        *reinterpret_cast<fused::u32x4_t*>(sv[stage] + (c * 8 + (v_kb ^ vswz(c))) * 16) = o;
      }
    }
  };

  fetch(0);
  stash(0);
  __syncthreads();
  for (int t = 0; t < ntiles; ++t) {
    const int cur = t & 1;
    const bool more = t + 1 < ntiles;
    if (more) fetch(t + 1);
    // ---- S^T = K Q^T for the 64 keys of the tile
    floatx16_t sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[mb][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const int row = mb * 32 + lr, c = kk * 2 + lh;
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sk[cur] + (row * C::CH + (c ^ C::kswz(row))) * 16);
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[mb], 0, 0, 0);
      }
    // ---- online softmax for this lane's query (keys: mb*32 + 8*(r/4) + 4*lh + r%4).
    //      The running maximum is kept in raw score units; the scale is folded into the
    //      exponent: p = 2^(s * scale2 - m * scale2).  Only tiles that reach a query's own
    //      position need the causal mask (a wave-uniform test).
    const int kv0 = t * BKV;
    float mx = -INFINITY;
    if (kv0 + BKV - 1 > qpos_min) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + mb * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
          if (key > qpos) sacc[mb][r] = -INFINITY;
        }
    }
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mb][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);          // finite from the first tile on (key 0 is visible)
    const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
    const float mneg = -m_new * scale2;
    float lsum = 0.f;
    bf16x8_t pf[4];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][r], scale2, mneg));
        lsum += p;
        pf[mb * 2 + (r >> 3)][r & 7] = (__bf16)p;
      }
    l_run = l_run * corr + lsum;
    m_run = m_new;
    if (__any(corr != 1.0f)) {            // the running maxima settle quickly: usually nothing to rescale
#pragma unroll
      for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] *= corr;
    }
    // ---- O^T += V^T P^T : k-step ts covers keys 16 ts .. 16 ts + 15 in slot order
    //      (lane half lh, element e) <-> key 16 ts + 4 lh + (e < 4 ? e : e + 4)
#pragma unroll
    for (int ts = 0; ts < 4; ++ts)
#pragma unroll
      for (int cb = 0; cb < C::CB; ++cb) {
        const int c = cb * 32 + lr;
        const char* rowp = sv[cur] + c * 128;
        const int ch0 = (2 * ts) ^ vswz(c), ch1 = (2 * ts + 1) ^ vswz(c);
        const uint2 lo = *reinterpret_cast<const uint2*>(rowp + ch0 * 16 + lh * 8);
        const uint2 hi = *reinterpret_cast<const uint2*>(rowp + ch1 * 16 + lh * 8);
        fused::u32x4_t vv = {lo.x, lo.y, hi.x, hi.y};
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, vv);
        oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ts], oacc[cb], 0, 0, 0);
      }
    if (more) stash(cur ^ 1);
    __syncthreads();
  }
  // ---- finish: this lane holds query qi, head dims cb*32 + 8*(r/4) + 4*lh + r%4
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < a.T_q) {
    const float inv = 1.0f / l_tot;
    const int64_t ob = ((int64_t)qi * a.H_q + h) * HD;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int c = cb * 32 + r4 * 8 + lh * 4;
        const float x0 = oacc[cb][r4 * 4] * inv, x1 = oacc[cb][r4 * 4 + 1] * inv;
        const float x2 = oacc[cb][r4 * 4 + 2] * inv, x3 = oacc[cb][r4 * 4 + 3] * inv;
        if (a.out_bf16) {
          uint2 w;
          w.x = (uint32_t)f32_to_bf16(x0) | ((uint32_t)f32_to_bf16(x1) << 16);
          w.y = (uint32_t)f32_to_bf16(x2) | ((uint32_t)f32_to_bf16(x3) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(a.out) + ob + c) = w;
        } else {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.out) + ob + c) = make_float4(x0, x1, x2, x3);
        }
      }
    if (a.lse && lh == 0)
      a.lse[(int64_t)qi * a.H_q + h] = (m_run * scale2 + __log2f(l_tot)) * 0.69314718055994530942f;
  }
}

}  // namespace prefill

template <typename T> inline bool prefill_mfma_supported(int d) {
  return sizeof(T) == 2 && (d == 64 || d == 128);
}

// k_ret / v_ret: retained cache at the sequence's first row (stride m);
// k_hat / v_hat: predicted dims of tokens 0 .. q_pos0+T_q-1 (stride d_out).
template <typename T>
inline int launch_prefill_mfma(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                               float scale, bool out_bf16,
                               const T* k_ret, const T* v_ret, const T* k_hat, const T* v_hat,
                               const T* q, int T_q, int q_pos0, void* out, float* lse,
                               hipStream_t st) {
  if constexpr (sizeof(T) != 2) {
    return 6;
  } else {
    prefill::Args a;
    a.k_ret = k_ret; a.v_ret = v_ret; a.k_hat = k_hat; a.v_hat = v_hat; a.q = q;
    a.out = out; a.lse = lse;
    a.H_q = H_q; a.G = H_q / H_kv; a.m = m; a.d_out = d_out; a.n_ret_heads = n_ret_heads;
    a.T_q = T_q; a.q_pos0 = q_pos0; a.out_bf16 = out_bf16 ? 1 : 0; a.scale = scale;
    dim3 grid((T_q + prefill::BQ - 1) / prefill::BQ, H_q);
    if (d == 128) hipLaunchKernelGGL((prefill::prefill_attn_kernel<128>), grid, dim3(prefill::NTHREADS), 0, st, a);
    else hipLaunchKernelGGL((prefill::prefill_attn_kernel<64>), grid, dim3(prefill::NTHREADS), 0, st, a);
    if (hipGetLastError() != hipSuccess) return 7;
    return 0;
  }
}

}  // namespace echokv
