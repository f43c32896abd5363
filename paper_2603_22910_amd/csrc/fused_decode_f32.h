// Fused reconstruct-then-attend decode kernel for an fp32 cache (gfx950).
//
// Same plan as the bf16 kernel (256 tokens x 256 predicted columns per
// workgroup, K pass with W as the row operand, V pass with X as the row
// operand, identical accumulator layout and therefore the same attention
// epilogues), but the predictor product (Eq. 3) runs on v_mfma_f32_32x32x2f32:
// true fp32 products and fp32 accumulation, as the 1e-5 tolerance of the fp32
// configuration needs.  An fp32 MFMA operand is ONE value per lane (row or
// column = lane % 32, k = lane / 32), so both tiles are read from LDS in their
// natural layouts with scalar reads and W needs no transposition.  The main
// loop is single-buffered and synchronous: this path exists for correctness on
// small fp32 problems, not for speed.
#pragma once
#include "common.h"
#include "fused_decode.h"

namespace echokv {
namespace fused32 {

using fused::BM; using fused::BN; using fused::NTHREADS; using fused::WM; using fused::WN;
constexpr int BK = 16;            // input dims per tile
constexpr int XP = BK + 1;        // padded row pitch of the X tile (floats): conflict-free column reads

struct Args {
  const float* xa[2]; const float* xr[2]; const float* w[2];
  const float* q;
  float* part_o; float* part_ml;
  int32_t D, m, d_out, H_q, G, n_ret_heads;
  float scale;
  int32_t n_col_tiles, n_tiles;
  const float* rope_cos; const float* rope_sin;     // rotary tables, or null
  int32_t n_sink, n_recent;                         // uncompressed window (0, 0: none)
};

struct Smem {
  float x[BM * XP];
  float w[BK * BN];
  fused::EpiSmem e;
};

template <bool SWAP>
__device__ __forceinline__ void gemm_pass(floatx16_t (&acc)[4][4], Smem& sm, const Args& a,
                                          const float* xa_tile, const float* xr_tile,
                                          const float* w_tile, int last, int n0, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1, lr = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int nk = (a.D + a.m) / BK, nka = a.D / BK;
  for (int kt = 0; kt < nk; ++kt) {
    const bool anchor = kt < nka;
    const float* xb = anchor ? xa_tile + kt * BK : xr_tile + (kt - nka) * BK;
    const int64_t ld = anchor ? a.D : a.m;
    float4 xs[4], ws[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = i * NTHREADS + tid, row = min(idx >> 2, last), c4 = idx & 3;
      xs[i] = *reinterpret_cast<const float4*>(xb + row * ld + c4 * 4);
      const int k = idx >> 6, n4 = idx & 63;
      const int n = min(n0 + n4 * 4, a.d_out - 4) - n0;      // clamp onto the last valid 4 columns
      ws[i] = *reinterpret_cast<const float4*>(w_tile + (int64_t)(kt * BK + k) * a.d_out + n);
    }
    __syncthreads();                      // previous tile fully consumed
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = i * NTHREADS + tid, row = idx >> 2, c4 = idx & 3;
      float* xd = &sm.x[row * XP + c4 * 4];
      xd[0] = xs[i].x; xd[1] = xs[i].y; xd[2] = xs[i].z; xd[3] = xs[i].w;
      const int k = idx >> 6, n4 = idx & 63;
      *reinterpret_cast<float4*>(&sm.w[k * BN + n4 * 4]) = ws[i];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < BK / 2; ++ks) {
      float xf[4], wf[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        xf[i] = sm.x[(wt * WM + i * 32 + lr) * XP + ks * 2 + lh];
        wf[i] = sm.w[(ks * 2 + lh) * BN + wc * WN + i * 32 + lr];
      }
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if constexpr (SWAP) acc[p][r] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[p], xf[r], acc[p][r], 0, 0, 0);
          else acc[p][r] = __builtin_amdgcn_mfma_f32_32x32x2f32(xf[p], wf[r], acc[p][r], 0, 0, 0);
        }
    }
  }
  __syncthreads();
}

template <int HD, bool ROPE>
__global__ __launch_bounds__(NTHREADS) void fused_decode_f32_kernel(Args a, SeqMeta meta) {
  __shared__ Smem sm;
  const int logical = blockIdx.x;
  const int ttile = logical / a.n_col_tiles, ctile = logical % a.n_col_tiles;
  const int b = find_seq(meta.tbase, meta.n, ttile);
  const int L = meta.len[b];
  const int j0 = (ttile - meta.tbase[b]) * BM;
  const int n0 = ctile * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1;
  const int last = min(BM, L - j0) - 1;
  const int64_t row0 = meta.start[b] + j0;
  fused::load_queries<HD>(sm.e, a.q, b, a.H_q, a.G, a.n_ret_heads + n0 / HD, a.scale, tid);
  floatx16_t acc[4][4];
  gemm_pass<true>(acc, sm, a, a.xa[0] + row0 * a.D, a.xr[0] + row0 * a.m, a.w[0] + n0, last, n0, tid);
  const int jw0 = j0 + wt * WM;
  fused::k_epilogue<HD, ROPE>(acc, sm.e, a.G, wave, lane, jw0, L,
                        fused::make_kextra(a.rope_cos, a.rope_sin, a.n_sink, a.n_recent, L));
  gemm_pass<false>(acc, sm, a, a.xa[1] + row0 * a.D, a.xr[1] + row0 * a.m, a.w[1] + n0, last, n0, tid);
  if (jw0 >= L) return;
  fused::v_epilogue<HD>(acc, sm.e, a.G, wave, lane, meta.sbase[b] + jw0 / kSlotTokens, a.H_q,
                        a.n_ret_heads + (n0 + wc * WN) / HD, a.part_o, a.part_ml);
}

}  // namespace fused32

inline int launch_fused_decode_f32(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                                   float scale, const float* ka,
                                   const float* va, const float* kr, const float* vr,
                                   const float* wk, const float* wv, const float* q,
                                   float* part_o, float* part_ml, SeqMeta& mt, int* fused_step,
                                   hipStream_t st, const KvExtras& ex = KvExtras()) {
  fused32::Args a;
  a.rope_cos = ex.rope_cos; a.rope_sin = ex.rope_sin; a.n_sink = ex.n_sink; a.n_recent = ex.n_recent;
  a.xa[0] = ka; a.xa[1] = va; a.xr[0] = kr; a.xr[1] = vr; a.w[0] = wk; a.w[1] = wv;
  a.q = q; a.part_o = part_o; a.part_ml = part_ml;
  a.D = H_kv * d; a.m = m; a.d_out = d_out; a.H_q = H_q; a.G = H_q / H_kv;
  a.n_ret_heads = n_ret_heads; a.scale = scale;
  a.n_col_tiles = (a.d_out + fused::BN - 1) / fused::BN;
  a.n_tiles = fused_fill_tiles(mt) * a.n_col_tiles;
  const dim3 g(a.n_tiles), blk(fused::NTHREADS);
  const bool rope = ex.rope_cos != nullptr;
  if (d == 128 && rope) hipLaunchKernelGGL((fused32::fused_decode_f32_kernel<128, true>), g, blk, 0, st, a, mt);
  else if (d == 128) hipLaunchKernelGGL((fused32::fused_decode_f32_kernel<128, false>), g, blk, 0, st, a, mt);
  else if (rope) hipLaunchKernelGGL((fused32::fused_decode_f32_kernel<64, true>), g, blk, 0, st, a, mt);
  else hipLaunchKernelGGL((fused32::fused_decode_f32_kernel<64, false>), g, blk, 0, st, a, mt);
  if (hipGetLastError() != hipSuccess) return 7;
  *fused_step = 1;
  return 0;
}

}  // namespace echokv
