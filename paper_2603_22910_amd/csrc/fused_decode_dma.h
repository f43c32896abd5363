// Fused reconstruct-then-attend decode kernel, direct-to-LDS variant (gfx950, bf16).
//
// Same tile (256 tokens x 256 predicted columns, 2 x 2 waves of 128 x 128), same
// MFMA formulation and the same attention epilogues as fused_decode_kernel, but
// the operand tiles travel HBM/L2 -> LDS with `buffer_load_dwordx4 ... lds`
// (no staging registers, no ds_write, no register transposes).  That needs both
// operands k-contiguous in memory, so this kernel takes the weights in the
// packed [d_out, d_in] layout of echokv_pack_weights.
//
// Pipeline: k-tiles of 32 input dims, FOUR LDS stages (4 x (16 KB X + 16 KB W)),
// three tiles in flight.  Per k-tile a wave issues its 8 loads of tile t+3,
// multiplies k-step 0 of tile t, waits until at most the 16 loads of tiles
// t+2 / t+3 are outstanding (so tile t+1 has landed), meets the other waves at
// one s_barrier, and multiplies k-step 1 while it reads the first fragments of
// tile t+1.  The barrier is a bare s_barrier: a full fence would make every
// wave wait for ALL its outstanding loads and serialise the prefetch.
#pragma once
#include "common.h"
#include "fused_decode.h"

namespace echokv {
namespace fdma {

using fused::BM; using fused::BN; using fused::NTHREADS; using fused::WM; using fused::WN;
using fused::Args; using fused::Frags; using fused::EpiSmem; using fused::rsrc_t;
constexpr int BK = 32;                       // input dims per k-tile
constexpr int NST = 4;                       // LDS stages
constexpr int kTileBytes = BM * BK * 2;      // 16 KB per operand per stage
#define ECHOKV_LDS __attribute__((address_space(3)))

// LDS tile: [256 rows][32 k] bf16, a row is 4 chunks of 16 bytes; chunk c of
// row r sits at slot c ^ ((r >> 2) & 3): 16 consecutive rows reading one chunk
// index touch 16 different 16-byte bank groups.
struct Lane {
  uint32_t fx[2], fw[2];   // fragment byte offsets for k-step 0 / 1 (block i adds i * 2048)
  uint32_t xrow[4];        // (clamped) tile row of this lane's X load i
  uint32_t vw[4];          // global byte offset of this lane's W^T load i
  uint32_t chunk;          // byte offset of this lane's 16-byte chunk inside a 64-byte k-slab
};

__device__ __forceinline__ void make_lane(Lane& ln, int tid, int last, int wlast, int D, int m,
                                          int d_in) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1, lr = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const uint32_t o = (uint32_t)(lr * 64 + (((2 * kk + lh) ^ ((lr >> 2) & 3)) << 4));
    ln.fx[kk] = o + wt * (WM * 64);
    ln.fw[kk] = o + wc * (WN * 64);
  }
  // load i of this wave fills rows (4 wave + i) * 16 + lane / 4; lane % 4 is the LDS
  // slot, which holds global chunk slot ^ ((row >> 2) & 3) = (lane & 3) ^ ((lane >> 4) & 3)
  ln.chunk = (uint32_t)((lane & 3) ^ ((lane >> 4) & 3)) * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (4 * wave + i) * 16 + (lane >> 2);
    ln.xrow[i] = (uint32_t)min(row, last);
    ln.vw[i] = __umul24(min(row, wlast), (uint32_t)d_in * 2) + ln.chunk;
  }
}

struct Stages {
  char* x[NST];
  char* w[NST];
};

struct Io {
  const bf16_t* pa;      // anchor rows of the tile (uniform)
  const bf16_t* pr;      // retained rows of the tile
  const bf16_t* pw;      // packed weights, row n0
  uint32_t D2, m2;       // row pitches in bytes
  int nk, nka, rot;
  __device__ __forceinline__ int ktile(int i) const {
    const int t = min(i, nk - 1) + rot;
    return t >= nk ? t - nk : t;
  }
};

// Issue this wave's 8 direct-to-LDS loads of k-tile `kn` into stage S.
template <int S>
__device__ __forceinline__ void dma_tile(const Stages& st, const Lane& ln, const Io& io, int kn,
                                         int wave_u) {
  // anchor dims first, then retained dims (Eq. 3): uniform selects, no branch
  const bool anchor = kn < io.nka;
  const rsrc_t rx = fused::make_rsrc(anchor ? io.pa : io.pr);
  const uint32_t ld2 = anchor ? io.D2 : io.m2;
  const int soff = (anchor ? kn : kn - io.nka) * (BK * 2);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (ECHOKV_LDS void*)(st.x[S] + (4 * wave_u + i) * 1024), 16,
                                             __umul24(ln.xrow[i], ld2) + ln.chunk, soff, 0, 0);
  const rsrc_t rw = fused::make_rsrc(io.pw);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (ECHOKV_LDS void*)(st.w[S] + (4 * wave_u + i) * 1024), 16,
                                             ln.vw[i], kn * (BK * 2), 0, 0);
}

template <int S>
__device__ __forceinline__ void read_frags(Frags& f, const Stages& st, const Lane& ln, int kk) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f.x[i] = *reinterpret_cast<const bf16x8_t*>(st.x[S] + ln.fx[kk] + i * 2048);
    f.w[i] = *reinterpret_cast<const bf16x8_t*>(st.w[S] + ln.fw[kk] + i * 2048);
  }
}

// wait until at most `n` of this wave's loads are outstanding, then meet the other waves
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));   // vmcnt(N), expcnt/lgkmcnt untouched
  __builtin_amdgcn_s_waitcnt(0xC07F);                                   // lgkmcnt(0): own LDS reads done
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <bool SWAP, int S>
__device__ __forceinline__ void k_tile(floatx16_t (&acc)[4][4], Frags& f0, Frags& f1,
                                       const Stages& st, const Lane& ln, const Io& io, int kfetch,
                                       int wave_u) {
  // tile t+3 -> the stage tile t-1 used (nobody reads it any more: its last
  // fragment reads were complete before the barrier inside tile t-1)
  dma_tile<(S + 3) % NST>(st, ln, io, kfetch, wave_u);
  read_frags<S>(f1, st, ln, 1);
  fused::mma16<SWAP>(acc, f0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(fused::SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(fused::SG_DS_RD, 1, 0);
    __builtin_amdgcn_sched_group_barrier(fused::SG_MFMA, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x10, 1, 0);     // one VMEM (the LDS-direct load)
  }
  __builtin_amdgcn_sched_barrier(0);
  wait_loads_and_barrier<16>();          // tile t+1 is in LDS for every wave
  read_frags<(S + 1) % NST>(f0, st, ln, 0);
  fused::mma16<SWAP>(acc, f1);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    __builtin_amdgcn_sched_group_barrier(fused::SG_MFMA, 2, 0);
    __builtin_amdgcn_sched_group_barrier(fused::SG_DS_RD, 1, 0);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Start a pass: three tiles in flight.
__device__ __forceinline__ void pass_begin(const Stages& st, const Lane& ln, const Io& io, int wave_u) {
  dma_tile<0>(st, ln, io, io.ktile(0), wave_u);
  dma_tile<1>(st, ln, io, io.ktile(1), wave_u);
  dma_tile<2>(st, ln, io, io.ktile(2), wave_u);
}

template <bool SWAP>
__device__ __forceinline__ void pass_run(floatx16_t (&acc)[4][4], const Stages& st, const Lane& ln,
                                         const Io& io, int wave_u) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  Frags f0, f1;
  wait_loads_and_barrier<16>();          // tile 0 has landed
  read_frags<0>(f0, st, ln, 0);
  const int nk = io.nk;
  int t = 0;
  for (; t + 4 <= nk; t += 4) {
    k_tile<SWAP, 0>(acc, f0, f1, st, ln, io, io.ktile(t + 3), wave_u);
    k_tile<SWAP, 1>(acc, f0, f1, st, ln, io, io.ktile(t + 4), wave_u);
    k_tile<SWAP, 2>(acc, f0, f1, st, ln, io, io.ktile(t + 5), wave_u);
    k_tile<SWAP, 3>(acc, f0, f1, st, ln, io, io.ktile(t + 6), wave_u);
  }
  if (t < nk) {       // d_in is a multiple of 64, so exactly two tiles are left
    k_tile<SWAP, 0>(acc, f0, f1, st, ln, io, io.ktile(t + 3), wave_u);
    k_tile<SWAP, 1>(acc, f0, f1, st, ln, io, io.ktile(t + 4), wave_u);
  }
  wait_loads_and_barrier<0>();           // drain: the stages are free for the next pass
}

template <int HD, bool ROPE>
__global__ __launch_bounds__(NTHREADS) void fused_decode_dma_kernel(Args a, SeqMeta meta) {
  __shared__ __attribute__((aligned(1024))) char sx0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sx1[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sx2[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sx3[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sw0[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sw1[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sw2[kTileBytes];
  __shared__ __attribute__((aligned(1024))) char sw3[kTileBytes];
  __shared__ EpiSmem epi;
  Stages st;
  st.x[0] = sx0; st.x[1] = sx1; st.x[2] = sx2; st.x[3] = sx3;
  st.w[0] = sw0; st.w[1] = sw1; st.w[2] = sw2; st.w[3] = sw3;
  int ttile, ctile;
  if (!fused::tile_of_block(a, ttile, ctile)) return;
  const int b = find_seq(meta.tbase, meta.n, ttile);
  const int L = meta.len[b];
  const int j0 = (ttile - meta.tbase[b]) * BM;
  const int n0 = ctile * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int wt = wave >> 1, wc = wave & 1;
  const int last = min(BM, L - j0) - 1;
  const int64_t row0 = meta.start[b] + j0;
  const int d_in = a.D + a.m;
  const int wlast = min(BN, a.d_out - n0) - 1;
  fused::load_queries<HD>(epi, a.q, b, a.H_q, a.G, a.n_ret_heads + n0 / HD, a.scale, tid);

  Lane ln;
  make_lane(ln, tid, last, wlast, a.D, a.m, d_in);
  Io io;
  io.nk = d_in / BK; io.nka = a.D / BK; io.rot = (ttile * 5) % io.nk;
  floatx16_t acc[4][4];
  // ---- K_hat^T = W_K^T X^T
  io.D2 = (uint32_t)a.D * 2; io.m2 = (uint32_t)a.m * 2;
  io.pa = a.xa[0] + row0 * a.D; io.pr = a.xr[0] + row0 * a.m; io.pw = a.w[0] + (int64_t)n0 * d_in;
  pass_begin(st, ln, io, wave_u);
  pass_run<true>(acc, st, ln, io, wave_u);          // its first barrier also publishes epi.q
  // the V pass's first three tiles are requested now and land during the score epilogue
  io.pa = a.xa[1] + row0 * a.D; io.pr = a.xr[1] + row0 * a.m; io.pw = a.w[1] + (int64_t)n0 * d_in;
  pass_begin(st, ln, io, wave_u);
  const int jw0 = j0 + wt * WM;
  fused::k_epilogue<HD, ROPE>(acc, epi, a.G, wave, lane, jw0, L,
                        fused::make_kextra(a.rope_cos, a.rope_sin, a.n_sink, a.n_recent, L));
  // ---- V_hat = X W_V
  pass_run<false>(acc, st, ln, io, wave_u);
  if (jw0 >= L) return;
  fused::v_epilogue<HD>(acc, epi, a.G, wave, lane, meta.sbase[b] + jw0 / kSlotTokens, a.H_q,
                        a.n_ret_heads + (n0 + wc * WN) / HD, a.part_o, a.part_ml);
}

}  // namespace fdma

inline int launch_fused_decode_dma(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                                   float scale, const bf16_t* ka, const bf16_t* va,
                                   const bf16_t* kr, const bf16_t* vr, const bf16_t* wk_packed,
                                   const bf16_t* wv_packed, const bf16_t* q, float* part_o,
                                   float* part_ml, SeqMeta& mt, int* fused_step, hipStream_t st,
                                   const KvExtras& ex = KvExtras()) {
  fused::Args a;
  a.rope_cos = ex.rope_cos; a.rope_sin = ex.rope_sin; a.n_sink = ex.n_sink; a.n_recent = ex.n_recent;
  a.s_out = nullptr; a.s_ld = 0;
  a.xa[0] = ka; a.xa[1] = va; a.xr[0] = kr; a.xr[1] = vr; a.w[0] = wk_packed; a.w[1] = wv_packed;
  a.q = q; a.part_o = part_o; a.part_ml = part_ml;
  a.out[0] = a.out[1] = nullptr; a.ldo = 0; a.col0 = 0;
  a.D = H_kv * d; a.m = m; a.d_out = d_out; a.H_q = H_q; a.G = H_q / H_kv;
  a.n_ret_heads = n_ret_heads; a.scale = scale;
  a.n_col_tiles = (a.d_out + fused::BN - 1) / fused::BN;
  a.n_tiles = fused_fill_tiles(mt) * a.n_col_tiles;
  const dim3 g(((a.n_tiles + 7) / 8) * 8), blk(fused::NTHREADS);
  const bool rope = ex.rope_cos != nullptr;
  if (d == 128 && rope) hipLaunchKernelGGL((fdma::fused_decode_dma_kernel<128, true>), g, blk, 0, st, a, mt);
  else if (d == 128) hipLaunchKernelGGL((fdma::fused_decode_dma_kernel<128, false>), g, blk, 0, st, a, mt);
  else if (rope) hipLaunchKernelGGL((fdma::fused_decode_dma_kernel<64, true>), g, blk, 0, st, a, mt);
  else hipLaunchKernelGGL((fdma::fused_decode_dma_kernel<64, false>), g, blk, 0, st, a, mt);
  if (hipGetLastError() != hipSuccess) return 7;
  *fused_step = 1;
  return 0;
}

}  // namespace echokv
