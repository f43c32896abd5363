// Weight-absorbed decode (gfx950, bf16 caches): the same attention output as
// reconstruct-then-attend, evaluated in the other association order.
//
// The predictor is linear (Eq. 3) and, in this library's cache model, nothing
// sits between reconstruction and the dot products of Eq. 7.  So with
// x_j = [anchor_j ; retained_j] (length d_in) and, per query head h of KV head g,
//     u_h[k] = sum_i Wt_K[k, g*d + i] q_h[i]        (Wt = W with the retained dims'
//                                                    selector columns put back, Eq. 6)
// the score is  s_j = x^K_j . u_h,  and the output is
//     o_h[i] = sum_k ( sum_j p_j x^V_j[k] ) Wt_V[k, g*d + i].
// Both token-sized products are skinny GEMMs (N = number of query heads) that
// read every cache row exactly once: the path is HBM-bound, not MFMA-bound.
//
// Kernels (all launched back to back on the caller's stream):
//   absorb_q      u = Wt_K q                       reads W_K once
//   scores        S^T[h, j] = u_h . x^K_j          streams the K caches, MFMA
//   softmax_stats per token split: M = max_j S, l = sum_j 2^(S - M)
//   pv            Y_part[h, k] = sum_j 2^(S - M) x^V_j[k]   streams the V caches, MFMA
//   y_sum         Y = merge of the splits' Y_part, normalised
//   out_partial   O_part = Y Wt_V over a slice of k     reads W_V once
//   out_final     out = sum of the slices
// Both streaming loops move whole row segments (512 contiguous bytes per row):
// the score pass through LDS, because its MFMA operand wants one token row per
// lane; the value pass straight into registers, where 8 x 8 blocks are
// transposed with byte permutes (the MFMA k-slot order is free as long as both
// operands agree).
#pragma once
#include "common.h"
#include "fused_decode.h"
#include "stream_kernels.h"

namespace echokv {
namespace absorbed {

using fused::rsrc_t; using fused::make_rsrc; using fused::u32x4_t;

constexpr int kHB = 32;           // query heads per MFMA block
constexpr int kTokTile = kSlotTokens;   // tokens per workgroup of the score pass
constexpr int kColTile = 256;     // predictor-input columns per workgroup of the value pass
constexpr int kPvWaves = 4;

struct Args {
  const bf16_t* xa[2];   // anchor cache K, V      [pool, D]
  const bf16_t* xr[2];   // retained cache K, V    [pool, m]
  const bf16_t* w[2];    // W_K, W_V               [D + m, d_out] row-major
  const bf16_t* q;       // [nseq, H_q, d]
  bf16_t* u;             // [nseq, H_pad, d_in]    absorbed queries, log2 units
  float* s;              // [H_pad, s_ld]          scores, log2 units; column = slot * 128 + token
  float* ml;             // [splits, H_pad, 2]     (max, sum) of each token split
  float* ypart;          // [splits, H_pad, d_in]
  float* y;              // [nseq, H_q, d_in]      normalised
  float* opart;          // [k_slices, nseq, H_q, d]
  float* y_ml;           // [nseq, H_q, 2]         (max in base-2 units, sum) of the merged splits
  // uncompressed window (value-absorbed mode only): its tokens are left out of the statistics
  // and the value pass, and its own partial (natural-exponent units, unnormalised o) joins at the end
  Window win;
  const float* win_po;   // [nseq, H_q, d] or null
  const float* win_pml;  // [nseq, H_q, 2]
  void* out; float* lse;
  int64_t out_seq0;
  int32_t D, m, d_in, d_out, H_q, H_pad, G, d;
  int32_t s_ld, split_tokens, n_col_a, n_col_tiles, k_slices, k_slice;
  int32_t single_split;  // every sequence is one token split: the value pass writes y and y_ml itself
  float qscale;          // softmax scale * log2(e)
};

// Element (k, f) of Wt: W[k, f - m] for a predicted dim f >= m, else the selector of
// retained dim f (input row D + f).
__device__ __forceinline__ void wt_row8(const bf16_t* w, int k, int f0, int m, int D, int d_out,
                                        float (&o)[8]) {
  if (f0 >= m) {
    load16<bf16_t>(w + (int64_t)k * d_out + (f0 - m), o);
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (k == D + f0 + i) ? 1.f : 0.f;
  }
}

// ---------------------------------------------------------------------------
// u[b, h, k] = qscale * sum_i Wt_K[k, g*d + i] q[b, h, i]   (bf16), on MFMA:
// C[pair, k] += Q[pair, i] Wt[k, i] with 32 (sequence, head-of-group) pairs as rows.
// grid = (ceil(d_in / 128), H_kv), 4 waves of 32 input rows each; a wave keeps
// its d / 16 Wt fragments in registers and walks over the pairs.
// ---------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(256) void absorb_q_kernel(Args a, int nseq) {
  constexpr int NS = HD / 16;
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lh = lane >> 5, wave = tid >> 6;
  const int g = blockIdx.y;
  const int k = blockIdx.x * 128 + wave * 32 + lr;
  const int kc = min(k, a.d_in - 1);
  u32x4_t wf[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int f0 = g * HD + 16 * s + 8 * lh;
    if (f0 >= a.m) {
      wf[s] = *reinterpret_cast<const u32x4_t*>(a.w[0] + (int64_t)kc * a.d_out + (f0 - a.m));
    } else {               // selector columns of the retained dims (Eq. 6): bf16 ones at k == D + f
#pragma unroll
      for (int p = 0; p < 4; ++p)
        wf[s][p] = (kc == a.D + f0 + 2 * p ? 0x3F80u : 0u) | (kc == a.D + f0 + 2 * p + 1 ? 0x3F800000u : 0u);
    }
  }
  const int npairs = nseq * a.G;
  for (int p0 = 0; p0 < npairs; p0 += 32) {
    const int pair = p0 + lr;
    const bool ok = pair < npairs;
    const int pc = ok ? pair : 0;
    const bf16_t* qp = a.q + ((int64_t)(pc / a.G) * a.H_q + g * a.G + pc % a.G) * HD + 8 * lh;
    floatx16_t acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    u32x4_t qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s] = *reinterpret_cast<const u32x4_t*>(qp + 16 * s);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      u32x4_t qq = qf[s];
      if (!ok) qq = u32x4_t{0u, 0u, 0u, 0u};
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, qq),
                                                    __builtin_bit_cast(bf16x8_t, wf[s]), acc, 0, 0, 0);
    }
    if (k < a.d_in) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int pr = p0 + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (pr < npairs)
          a.u[((int64_t)(pr / a.G) * a.H_pad + g * a.G + pr % a.G) * a.d_in + k] = f32_to_bf16(acc[r] * a.qscale);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Score pass.  One workgroup (4 waves) = one 128-token slot of one sequence x
// one block of 32 query heads; wave w owns tokens 32 w .. 32 w + 31 for the
// whole of d_in, so no partial sums ever meet.  MFMA form:
// C[head, token] += U[head, k] X[token, k]: a lane owns a token column and the
// stores to S^T are 128-byte rows.
//
// The MFMA operand layout wants, per lane, 16 bytes of a different token row:
// loaded straight from global memory that is 32 rows x 32 bytes per
// instruction, a pattern that reaches barely half of the streaming bandwidth.
// So X and U go HBM / L2 -> LDS in stages of 128 input dims with
// `buffer_load ... lds` (one instruction = 4 rows x 256 contiguous bytes) and
// the fragments are read back from LDS (chunk c of row r sits at slot
// c ^ (r % 16): conflict-free 16-byte reads down a column).  Two stages of
// 40 KB, so two workgroups share a compute unit and cover each other's barriers.
// ---------------------------------------------------------------------------
#ifndef ECHOKV_LDS
#define ECHOKV_LDS __attribute__((address_space(3)))
#endif
constexpr int kStageK = 128;                              // input dims per LDS stage
constexpr int kRowBytes = kStageK * 2;                    // 256
constexpr int kXBytes = kTokTile * kRowBytes;             // 32 KB
constexpr int kUBytes = kHB * kRowBytes;                  // 8 KB
constexpr int kStageBytes = kXBytes + kUBytes;            // 40 KB

struct ScoreIo {
  const bf16_t* pa; const bf16_t* pr;
  rsrc_t ru;
  uint32_t D2, m2, u2;
  int D, m, nsa, ns, last;
  int rot;        // stage visited first: workgroups that run side by side read different columns
};

struct StageDesc { bool anchor; int k0, kw, kg0; };
__device__ __forceinline__ StageDesc stage_desc(const ScoreIo& io, int t) {
  t = min(t, io.ns - 1) + io.rot;
  if (t >= io.ns) t -= io.ns;
  StageDesc d;
  d.anchor = t < io.nsa;
  d.k0 = (d.anchor ? t : t - io.nsa) * kStageK;
  d.kw = min(kStageK, (d.anchor ? io.D : io.m) - d.k0);
  d.kg0 = d.anchor ? d.k0 : io.D + d.k0;
  return d;
}

// this wave's 10 direct-to-LDS loads of stage t: X rows 32 w .. 32 w + 31, U rows 8 w .. 8 w + 7
__device__ __forceinline__ void score_issue(char* buf, const ScoreIo& io, int t, int wave, int lane) {
  const StageDesc d = stage_desc(io, t);
  const rsrc_t rx = make_rsrc(d.anchor ? io.pa : io.pr);
  const uint32_t ld2 = d.anchor ? io.D2 : io.m2;
  const int nchunk = d.kw / 8;
  const int sub = lane >> 4, slot = lane & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = wave * 32 + 4 * i + sub;
    const int chunk = min(slot ^ (row & 15), nchunk - 1);            // a partial stage repeats its last chunk
    const uint32_t voff = __umul24((uint32_t)min(row, io.last), ld2) + (uint32_t)chunk * 16;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, (ECHOKV_LDS void*)(buf + (wave * 32 + 4 * i) * kRowBytes),
                                             16, voff, d.k0 * 2, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = wave * 8 + 4 * i + sub;
    const int chunk = min(slot ^ (row & 15), nchunk - 1);
    const uint32_t voff = __umul24((uint32_t)row, io.u2) + (uint32_t)chunk * 16;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(io.ru, (ECHOKV_LDS void*)(buf + kXBytes + (wave * 8 + 4 * i) * kRowBytes),
                                             16, voff, d.kg0 * 2, 0, 0);
  }
}

template <int NST>
__device__ __forceinline__ void score_wait_landed() {
  constexpr int N = 10 * (NST - 1);            // loads of the younger stages, which may stay in flight
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));     // vmcnt(N)
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}
__device__ __forceinline__ void score_wait_read() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0): own fragment reads returned
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int NST>
__device__ __forceinline__ void score_stage(floatx16_t& acc, char* buf, const ScoreIo& io, int t,
                                            int wave, int lane, bool head_ok) {
  const int lr = lane & 31, lh = lane >> 5;
  const StageDesc d = stage_desc(io, t);
  const int kw = (head_ok && t < io.ns) ? d.kw : 0;       // input dims of this stage that count
  score_wait_landed<NST>();                     // stage t is in LDS for every wave
  u32x4_t xf[8], uf[8];
  const char* xrow = buf + (wave * 32 + lr) * kRowBytes;
  const char* urow = buf + kXBytes + lr * kRowBytes;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int off = ((2 * s + lh) ^ (lr & 15)) << 4;
    xf[s] = *reinterpret_cast<const u32x4_t*>(xrow + off);
    uf[s] = *reinterpret_cast<const u32x4_t*>(urow + off);
  }
  score_wait_read();                            // every wave holds its fragments: the buffer is free
  score_issue(buf, io, t + NST, wave, lane);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    u32x4_t uu = uf[s];
    if (16 * s >= kw) uu = u32x4_t{0u, 0u, 0u, 0u};
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, uu),
                                                  __builtin_bit_cast(bf16x8_t, xf[s]), acc, 0, 0, 0);
  }
}

template <int NST>      // LDS stages: 2 (80 KB, two workgroups per compute unit) or 4 (160 KB, for small grids)
__global__ __launch_bounds__(256, NST == 2 ? 2 : 1) void scores_kernel(Args a, SeqMeta meta) {
  __shared__ __attribute__((aligned(1024))) char lds[NST * kStageBytes];
  const int slot = blockIdx.x, hb = blockIdx.y;
  const int b = find_seq(meta.sbase, meta.n, slot);
  const int L = meta.len[b];
  const int j0 = (slot - meta.sbase[b]) * kTokTile;
  const int64_t row0 = meta.start[b] + j0;
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  ScoreIo io;
  io.pa = a.xa[0] + row0 * a.D; io.pr = a.xr[0] + row0 * a.m;
  io.ru = make_rsrc(a.u + ((int64_t)b * a.H_pad + hb * kHB) * a.d_in);
  io.D2 = (uint32_t)a.D * 2; io.m2 = (uint32_t)a.m * 2; io.u2 = (uint32_t)a.d_in * 2;
  io.D = a.D; io.m = a.m;
  io.nsa = (a.D + kStageK - 1) / kStageK; io.ns = io.nsa + (a.m + kStageK - 1) / kStageK;
  io.last = min(kTokTile, L - j0) - 1;
  io.rot = (slot * 5) % io.ns;
  const bool head_ok = hb * kHB + lr < a.H_q;    // rows of U past the last head hold nothing: count as zero

  floatx16_t acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;

  // stage t lives in buffer t % NST; stages past the last one repeat it with U counted as
  // zero, so every wave runs the same barriers
#pragma unroll
  for (int i = 0; i < NST; ++i) score_issue(lds + i * kStageBytes, io, i, wave, lane);
  for (int t = 0; t < io.ns; t += NST) {
#pragma unroll
    for (int i = 0; i < NST; ++i) score_stage<NST>(acc, lds + i * kStageBytes, io, t + i, wave, lane, head_ok);
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): the look-ahead loads land before the block's LDS is released
  float* srow = a.s + (int64_t)slot * kTokTile + wave * 32 + lr;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int head = 8 * (r >> 2) + 4 * lh + (r & 3);      // accumulator row -> head
    srow[(int64_t)(hb * kHB + head) * a.s_ld] = acc[r];
  }
}

// ---------------------------------------------------------------------------
// (max, sum of 2^(S - max)) of one (token split, head) piece of a row of S^T, in one pass over
// the scores: every thread keeps a running (max, sum) pair over its elements, four independent
// chains per thread, and the pairs are merged exactly (sum' = sum 2^(max - max')).
// grid = (H_q, splits), NT threads.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void ml_push(float& M, float& l, float x) {
  const float Mn = fmaxf(M, x);                 // x is finite: Mn is finite from the first element on
  l = l * exp2f(M - Mn) + exp2f(x - Mn);        // (M = -inf: the old sum, 0, is scaled by 0)
  M = Mn;
}
__device__ __forceinline__ void ml_merge(float& M, float& l, float M2, float l2) {
  const float Mn = fmaxf(M, M2);
  const float w1 = M == -INFINITY ? 0.f : exp2f(M - Mn), w2 = M2 == -INFINITY ? 0.f : exp2f(M2 - Mn);
  l = l * w1 + l2 * w2;
  M = Mn;
}
template <int NT>
__global__ __launch_bounds__(NT) void softmax_stats_kernel(Args a, SeqMeta meta) {
  const int h = blockIdx.x, sp = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = find_seq(meta.tbase, meta.n, sp);
  const int t_begin = (sp - meta.tbase[b]) * a.split_tokens;
  const int L = meta.len[b];
  const int j0 = max(0, a.win.lo(L) - t_begin);                       // window tokens are left out
  const int n = min(min(L, a.win.hi(L)) - t_begin, a.split_tokens);   // (an empty piece gets (-inf, 0))
  const float* row = a.s + (int64_t)h * a.s_ld + (int64_t)meta.sbase[b] * kSlotTokens + t_begin;
  __shared__ float s_m[NT / 64], s_l[NT / 64];
  float M[4], l[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) { M[c] = -INFINITY; l[c] = 0.f; }
  int j = j0 + tid;
  for (; j + 3 * NT < n; j += 4 * NT) {
    float x[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) x[c] = row[j + c * NT];
#pragma unroll
    for (int c = 0; c < 4; ++c) ml_push(M[c], l[c], x[c]);
  }
  for (; j < n; j += NT) ml_push(M[0], l[0], row[j]);
#pragma unroll
  for (int c = 1; c < 4; ++c) ml_merge(M[0], l[0], M[c], l[c]);
  // over the wave, then over the waves
  const float Mw = wave_max(M[0], 64);
  float lw = M[0] == -INFINITY ? 0.f : l[0] * exp2f(M[0] - Mw);
  lw = wave_sum(lw, 64);
  if (lane == 0) { s_m[wave] = Mw; s_l[wave] = lw; }
  __syncthreads();
  if (tid == 0) {
    float Mt = s_m[0], lt = s_l[0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) ml_merge(Mt, lt, s_m[w], s_l[w]);
    float* ml = a.ml + ((int64_t)sp * a.H_pad + h) * 2;
    ml[0] = Mt; ml[1] = lt;
  }
}

// ---------------------------------------------------------------------------
// Value pass.  One workgroup = one token split of one sequence x 256 input
// columns (anchor columns or retained columns, never both) x 32 query heads;
// its 4 waves take every 4th step of 16 tokens.
// MFMA form: C[head, col] += P^T[head, token] X[token, col].  A lane loads, for
// 8 consecutive columns, the 8 token rows of its half (512-byte row segments
// across the wave), transposes the 8 x 8 block in registers and so owns
// column 8 * (lane % 32) + i of MFMA i.
// ---------------------------------------------------------------------------
struct PvStage {
  u32x4_t x[8];      // token lh * 8 + e, 8 columns
  u32x4_t s[2];      // 8 scores of head lane % 32
};

struct PvIo {
  rsrc_t rx, rs;
  uint32_t pitch2, colb, soff0;
  int nrows, nsteps;
  int lh8;
  int vlo, vhi;      // rows [vlo, vhi) of the split count (the others are past the end or in the window)
};

__device__ __forceinline__ void pv_fetch(PvStage& st, const PvIo& io, int step) {
  step = min(step, io.nsteps - 1);
  const int t0 = step * 16 + io.lh8;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t row = (uint32_t)min(t0 + e, io.nrows - 1);
    st.x[e] = __builtin_amdgcn_raw_buffer_load_b128(io.rx, __umul24(row, io.pitch2) + io.colb, 0, 0);
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
    st.s[i] = __builtin_amdgcn_raw_buffer_load_b128(io.rs, io.soff0 + i * 16, step * 64, 0);
}

__device__ __forceinline__ void pv_mma(floatx16_t (&acc)[8], const PvStage& st, const PvIo& io,
                                       int step, float M) {
  // probabilities of this lane's head for its 8 tokens (0 beyond the split's end)
  const int t0 = step * 16 + io.lh8;
  // each probability goes in as a bf16 (high, low) pair: the value pass is far from
  // MFMA-bound, and this keeps the rounding of p out of the result
  u32x4_t pw, pl;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float s0 = __uint_as_float(st.s[i >> 1][(2 * i) & 3]);
    const float s1 = __uint_as_float(st.s[i >> 1][(2 * i + 1) & 3]);
    const float p0 = (t0 + 2 * i >= io.vlo && t0 + 2 * i < io.vhi) ? exp2f(s0 - M) : 0.f;
    const float p1 = (t0 + 2 * i + 1 >= io.vlo && t0 + 2 * i + 1 < io.vhi) ? exp2f(s1 - M) : 0.f;
    const bf16_t h0 = f32_to_bf16(p0), h1 = f32_to_bf16(p1);
    pw[i] = (uint32_t)h0 | ((uint32_t)h1 << 16);
    pl[i] = (uint32_t)f32_to_bf16(p0 - bf16_to_f32(h0)) | ((uint32_t)f32_to_bf16(p1 - bf16_to_f32(h1)) << 16);
  }
  const bf16x8_t pa = __builtin_bit_cast(bf16x8_t, pw);
  const bf16x8_t pb = __builtin_bit_cast(bf16x8_t, pl);
  // 8 x 8 transpose: word p of output i holds tokens 2p, 2p + 1 of column i
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    u32x4_t xt;
#pragma unroll
    for (int p = 0; p < 4; ++p)
      xt[p] = __builtin_amdgcn_perm(st.x[2 * p + 1][i >> 1], st.x[2 * p][i >> 1],
                                    (i & 1) ? 0x07060302u : 0x05040100u);
    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa, __builtin_bit_cast(bf16x8_t, xt), acc[i], 0, 0, 0);
    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pb, __builtin_bit_cast(bf16x8_t, xt), acc[i], 0, 0, 0);
  }
}

__global__ __launch_bounds__(kPvWaves * 64, 2) void pv_kernel(Args a, SeqMeta meta) {
  __shared__ float red[2][128][64];       // 64 KB: two waves' accumulators
  const int ct = blockIdx.x % a.n_col_tiles, sp = blockIdx.x / a.n_col_tiles, hb = blockIdx.y;
  const int b = find_seq(meta.tbase, meta.n, sp);
  const int L = meta.len[b];
  const int t_begin = (sp - meta.tbase[b]) * a.split_tokens;
  const int nrows = min(L - t_begin, a.split_tokens);
  const bool anchor = ct < a.n_col_a;
  const int c0 = (anchor ? ct : ct - a.n_col_a) * kColTile;
  const int width = anchor ? a.D : a.m;
  const int64_t row0 = meta.start[b] + t_begin;
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = c0 + 8 * lr;
  const bool col_ok = col < width;

  PvIo io;
  io.rx = make_rsrc((anchor ? a.xa[1] : a.xr[1]) + row0 * width);
  io.rs = make_rsrc(a.s + (int64_t)hb * kHB * a.s_ld + (int64_t)meta.sbase[b] * kSlotTokens + t_begin);
  io.pitch2 = (uint32_t)width * 2;
  io.colb = (uint32_t)(col_ok ? col : 0) * 2;
  io.soff0 = ((uint32_t)lr * (uint32_t)a.s_ld + (uint32_t)lh * 8) * 4;
  io.nrows = nrows; io.nsteps = (nrows + 15) / 16; io.lh8 = lh * 8;
  io.vlo = max(0, a.win.lo(L) - t_begin); io.vhi = min(nrows, a.win.hi(L) - t_begin);
  const int head = hb * kHB + lr;
  float M = head < a.H_q ? a.ml[((int64_t)sp * a.H_pad + head) * 2] : 0.f;   // the split's own maximum
  if (M == -INFINITY) M = 0.f;                    // a piece with no counted token: every p is masked

  floatx16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  // two register stages, branch-free body: rounds past the wave's last step
  // re-read the split's last step with all probabilities masked to zero
  PvStage s0, s1;
  const int n = io.nsteps;
  const int nw = (n - wave + kPvWaves - 1) / kPvWaves;
  pv_fetch(s0, io, wave);
  for (int it = 0; it < nw; it += 2) {
    const int st = wave + it * kPvWaves;
    pv_fetch(s1, io, st + kPvWaves);
    pv_mma(acc, s0, io, st, M);
    pv_fetch(s0, io, st + 2 * kPvWaves);
    pv_mma(acc, s1, io, st + kPvWaves, M);
  }

  // tree reduction over the 4 waves: {2, 3} -> {0, 1}, then 1 -> 0
  if (wave >= 2) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[wave - 2][i * 16 + r][lane] = acc[i][r];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] += red[wave][i * 16 + r][lane];
  }
  __syncthreads();
  if (wave == 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[0][i * 16 + r][lane] = acc[i][r];
  }
  __syncthreads();
  if (wave != 0) return;
  if (a.single_split && ct == 0 && lh == 0 && head < a.H_q) {     // the split is the sequence: its (max, sum) is final
    const float* ml = a.ml + ((int64_t)sp * a.H_pad + head) * 2;
    a.y_ml[((int64_t)b * a.H_q + head) * 2] = ml[0];
    a.y_ml[((int64_t)b * a.H_q + head) * 2 + 1] = ml[1];
  }
  if (!col_ok) return;
  float* yp = a.ypart + ((int64_t)sp * a.H_pad + hb * kHB) * a.d_in + (anchor ? 0 : a.D) + col;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int hr = 8 * (r >> 2) + 4 * lh + (r & 3);
    float4 lo, hi;
    lo.x = acc[0][r] + red[0][0 * 16 + r][lane]; lo.y = acc[1][r] + red[0][1 * 16 + r][lane];
    lo.z = acc[2][r] + red[0][2 * 16 + r][lane]; lo.w = acc[3][r] + red[0][3 * 16 + r][lane];
    hi.x = acc[4][r] + red[0][4 * 16 + r][lane]; hi.y = acc[5][r] + red[0][5 * 16 + r][lane];
    hi.z = acc[6][r] + red[0][6 * 16 + r][lane]; hi.w = acc[7][r] + red[0][7 * 16 + r][lane];
    float* dst = yp + (int64_t)hr * a.d_in;
    if (a.single_split) {       // normalised, straight into y (what y_sum would make of one split)
      const int ha = hb * kHB + hr;
      if (ha >= a.H_q) continue;
      const float l = a.ml[((int64_t)sp * a.H_pad + ha) * 2 + 1];
      const float inv = l > 0.f ? 1.f / l : 0.f;        // l == 0: every counted token sits in the window
      lo.x *= inv; lo.y *= inv; lo.z *= inv; lo.w *= inv; hi.x *= inv; hi.y *= inv; hi.z *= inv; hi.w *= inv;
      dst = a.y + ((int64_t)b * a.H_q + ha) * a.d_in + (anchor ? 0 : a.D) + col;
    }
    *reinterpret_cast<float4*>(dst) = lo;
    *reinterpret_cast<float4*>(dst + 4) = hi;
  }
}

// ---------------------------------------------------------------------------
// Merge of a sequence's token splits (exact re-association of the softmax):
//   M = max_s M_s,  l = sum_s l_s 2^(M_s - M),  y[b, h, k] = sum_s 2^(M_s - M) ypart_s[h, k] / l
// and (M, l) for the last kernel.  grid = (ceil(d_in / (1024 / SG)), H_q, nseq).
// ---------------------------------------------------------------------------
template <int SG>       // thread groups that share a column quad and split the splits: 1 (few splits) or 4
__global__ __launch_bounds__(256) void y_sum_kernel(Args a, SeqMeta meta) {
  constexpr int CQ = 256 / SG;                   // column quads per workgroup
  const int h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int cq = tid % CQ, sg = tid / CQ;
  const int k = min((blockIdx.x * CQ + cq) * 4, a.d_in - 4);     // tail threads repeat the last quad
  const int s0 = meta.tbase[b], ns = meta.tbase[b + 1] - s0;
  __shared__ float s_red[4];
  __shared__ float s_w[256];
  __shared__ float4 s_acc[SG][CQ];
  const float* mlp = a.ml + ((int64_t)s0 * a.H_pad + h) * 2;
  const int64_t mls = (int64_t)a.H_pad * 2;
  float M = -INFINITY;
  for (int i = tid; i < ns; i += 256) M = fmaxf(M, mlp[i * mls]);
  M = wave_max(M, 64);
  if (lane == 0) s_red[wave] = M;
  __syncthreads();
  M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float l = 0.f;
  const float* yp = a.ypart + ((int64_t)s0 * a.H_pad + h) * a.d_in + k;
  const int64_t yps = (int64_t)a.H_pad * a.d_in;
  for (int c0 = 0; c0 < ns; c0 += 256) {
    float wgt = 0.f;
    if (c0 + tid < ns) {
      const float ms = mlp[(c0 + tid) * mls];
      wgt = ms == -INFINITY ? 0.f : exp2f(ms - M);
      l += wgt * mlp[(c0 + tid) * mls + 1];
    }
    __syncthreads();            // the previous chunk's weights are no longer read
    s_w[tid] = wgt;
    __syncthreads();
    const int cn = min(256, ns - c0);
#pragma unroll 8
    for (int j = sg; j < cn; j += SG) {
      const float4 v = *reinterpret_cast<const float4*>(yp + (c0 + j) * yps);
      const float wj = s_w[j];
      acc.x = fmaf(wj, v.x, acc.x); acc.y = fmaf(wj, v.y, acc.y);
      acc.z = fmaf(wj, v.z, acc.z); acc.w = fmaf(wj, v.w, acc.w);
    }
  }
  l = wave_sum(l, 64);
  s_acc[sg][cq] = acc;
  __syncthreads();              // s_red was read above by every thread
  if (lane == 0) s_red[wave] = l;
  __syncthreads();
  if (sg != 0) return;
  l = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
  const float inv = l > 0.f ? 1.f / l : 0.f;       // l == 0: every counted token sits in the window
#pragma unroll
  for (int g = 1; g < SG; ++g) {
    acc.x += s_acc[g][cq].x; acc.y += s_acc[g][cq].y; acc.z += s_acc[g][cq].z; acc.w += s_acc[g][cq].w;
  }
  acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  *reinterpret_cast<float4*>(a.y + ((int64_t)b * a.H_q + h) * a.d_in + k) = acc;
  if (blockIdx.x == 0 && tid == 0) {
    a.y_ml[((int64_t)b * a.H_q + h) * 2] = M;
    a.y_ml[((int64_t)b * a.H_q + h) * 2 + 1] = l;
  }
}

// ---------------------------------------------------------------------------
// opart[ks, b, h, i] = sum over k in slice ks of y[b, h, k] Wt_V[k, g*d + i], on MFMA:
// C[pair, i] += Y[pair, k] Wt[k, i].  y goes in as a bf16 (high, low) pair, so
// the product keeps fp32-like accuracy.  The contraction runs down the rows of
// W_V, so a lane loads 8 rows x (d / 32) columns and transposes them in
// registers; it owns columns (d / 32) * (lane % 32) + i.
// grid = (H_kv, k_slices, ceil(nseq * G / 32)); the 4 waves take every 4th step
// of 16 input rows and meet in LDS.
// ---------------------------------------------------------------------------
template <int HD>
struct OutStage {
  uint32_t x[8][HD / 64];     // 8 input rows x (d / 32) bf16 columns
  float4 y[2];                // 8 consecutive y values of this lane's pair
};

template <int HD>
__global__ __launch_bounds__(256) void out_partial_kernel(Args a, int nseq) {
  constexpr int CPL = HD / 32, WPL = HD / 64;      // columns, 32-bit words per lane and row
  __shared__ float red[3][CPL * 16][64];
  const int g = blockIdx.x, ks = blockIdx.y, p0 = blockIdx.z * 32;
  const int tid = threadIdx.x, lane = tid & 63, lr = lane & 31, lh = lane >> 5, wave = tid >> 6;
  const int npairs = nseq * a.G;
  const int k0 = ks * a.k_slice, kn = min(a.k_slice, a.d_in - k0), nsteps = kn / 16;
  const int pair = p0 + lr;
  const bool ok = pair < npairs;
  const int pc = ok ? pair : 0;
  const float* yrow = a.y + ((int64_t)(pc / a.G) * a.H_q + g * a.G + pc % a.G) * a.d_in + k0 + lh * 8;
  const int f0 = g * HD + CPL * lr;
  const bool pred = f0 >= a.m;
  const bf16_t* wcol = a.w[1] + (int64_t)(k0 + lh * 8) * a.d_out + (pred ? f0 - a.m : 0);

  auto fetch = [&](OutStage<HD>& st, int step) {
    step = min(step, nsteps - 1);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int kk = step * 16 + e;
      if (pred) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(wcol + (int64_t)kk * a.d_out);
#pragma unroll
        for (int w = 0; w < WPL; ++w) st.x[e][w] = src[w];
      } else {
        const int kg = k0 + lh * 8 + kk;           // selector columns of the retained dims (Eq. 6)
#pragma unroll
        for (int w = 0; w < WPL; ++w)
          st.x[e][w] = (kg == a.D + f0 + 2 * w ? 0x3F80u : 0u) | (kg == a.D + f0 + 2 * w + 1 ? 0x3F800000u : 0u);
      }
    }
    st.y[0] = *reinterpret_cast<const float4*>(yrow + step * 16);
    st.y[1] = *reinterpret_cast<const float4*>(yrow + step * 16 + 4);
  };
  floatx16_t acc[CPL];
#pragma unroll
  for (int i = 0; i < CPL; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  auto mma = [&](const OutStage<HD>& st, bool live) {
    const float yv[8] = {st.y[0].x, st.y[0].y, st.y[0].z, st.y[0].w, st.y[1].x, st.y[1].y, st.y[1].z, st.y[1].w};
    u32x4_t hi, lo;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      uint32_t h2[2], l2[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const float v = live ? yv[2 * p + q] : 0.f;
        const bf16_t hb = f32_to_bf16(v);
        h2[q] = hb; l2[q] = f32_to_bf16(v - bf16_to_f32(hb));
      }
      hi[p] = h2[0] | (h2[1] << 16); lo[p] = l2[0] | (l2[1] << 16);
    }
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      u32x4_t xt;
#pragma unroll
      for (int p = 0; p < 4; ++p)
        xt[p] = __builtin_amdgcn_perm(st.x[2 * p + 1][i >> 1], st.x[2 * p][i >> 1],
                                      (i & 1) ? 0x07060302u : 0x05040100u);
      const bf16x8_t xb = __builtin_bit_cast(bf16x8_t, xt);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, hi), xb, acc[i], 0, 0, 0);
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, lo), xb, acc[i], 0, 0, 0);
    }
  };
  // four register stages: a slice of 256 input rows is 4 steps per wave, all in flight at once
  OutStage<HD> s0, s1, s2, s3;
  const int nw = (nsteps - wave + 3) / 4;
  for (int it = 0; it < nw; it += 4) {
    const int st = wave + it * 4;
    fetch(s0, st); fetch(s1, st + 4); fetch(s2, st + 8); fetch(s3, st + 12);
    mma(s0, ok);
    mma(s1, ok && it + 1 < nw);
    mma(s2, ok && it + 2 < nw);
    mma(s3, ok && it + 3 < nw);
  }
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < CPL; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) red[wave - 1][i * 16 + r][lane] = acc[i][r];
  }
  __syncthreads();
  if (wave > 0) return;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int pr = p0 + 8 * (r >> 2) + 4 * lh + (r & 3);
    if (pr >= npairs) continue;
    float* dst = a.opart + (((int64_t)ks * nseq + pr / a.G) * a.H_q + g * a.G + pr % a.G) * HD + CPL * lr;
#pragma unroll
    for (int i = 0; i < CPL; ++i)
      dst[i] = acc[i][r] + ((red[0][i * 16 + r][lane] + red[1][i * 16 + r][lane]) + red[2][i * 16 + r][lane]);
  }
}

// out[b, h, :] = sum over k slices of opart, joined with the window's partial if there is one
// (exact re-association of the softmax over {compressed tokens} + {window tokens}), and the
// log-sum-exp.  grid = ceil(nseq * H_q * d / 256).
template <typename TO>
__global__ __launch_bounds__(256) void out_final_kernel(Args a, int nseq) {
  const int64_t n = (int64_t)nseq * a.H_q * a.d;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n) return;
  float v = 0.f;
#pragma unroll 4
  for (int ks = 0; ks < a.k_slices; ++ks) v += a.opart[(int64_t)ks * n + idx];
  const int64_t bh = idx / a.d;
  const float M2 = a.y_ml[bh * 2], lY = a.y_ml[bh * 2 + 1];
  float M = lY > 0.f ? M2 * 0.6931471805599453f : -INFINITY;     // natural-exponent units
  float denom = lY;
  if (a.win_po) {
    const float mw = a.win_pml[bh * 2], lw = a.win_pml[bh * 2 + 1];
    const float Mn = fmaxf(M, mw);
    const float wy = lY > 0.f ? __expf(M - Mn) * lY : 0.f;
    const float ww = lw > 0.f ? __expf(mw - Mn) : 0.f;
    denom = wy + ww * lw;
    v = (wy * v + ww * a.win_po[idx]) / denom;
    M = Mn;
  }
  TO* out = (TO*)a.out + a.out_seq0 * a.H_q * a.d;
  if constexpr (sizeof(TO) == 2) out[idx] = f32_to_bf16(v);
  else out[idx] = v;
  if (a.lse && idx % a.d == 0) a.lse[a.out_seq0 * a.H_q + bh] = M + __logf(denom);
}

}  // namespace absorbed
}  // namespace echokv
