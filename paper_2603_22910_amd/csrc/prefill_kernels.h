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

#include <algorithm>

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
  // split over the keys (long-chunk kernel only; kv_splits == 1: off): workgroup z of a (head,
  // query block) takes one share of the block's key tiles and writes its unnormalised partial
  // instead of the output; prefill_merge_kernel joins the shares.
  int32_t kv_splits;
  float* part_o;                              // [T_q, H_q, kv_splits, d]
  float* part_ml;                             // [T_q, H_q, kv_splits, 2]: (max in base-2 units, sum)
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

// The softmax reference maximum of a query is raised only when the running maximum has moved
// more than kSlack above it (in base-2 exponent units): the probabilities then stay below
// 2^kSlack, harmless in fp32 / bf16, sums and outputs are exact either way, and the
// accumulators are rescaled once in a while instead of on most tiles.
constexpr float kSlack = 8.0f;
// max of a value over the two lanes (l, l + 32) that share a query, on the vector ALU
__device__ __forceinline__ float max_over_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int HD>
__global__ __launch_bounds__(NTHREADS, 2) void prefill_attn_kernel(Args a) {
  using C = Cfg<HD>;
  __shared__ __attribute__((aligned(16))) char sk[2][C::KTILE_BYTES];
  __shared__ __attribute__((aligned(16))) char sv[2][C::VTILE_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  // grid = (heads, query blocks): workgroups are handed out x first, so every head's longest
  // (latest) query block starts before any shorter one -- a causal chunk's work per block grows
  // linearly, and with the heads outermost the last head's longest blocks would start last
  const int h = blockIdx.x;
  const int nqb = (a.T_q + BQ - 1) / BQ;
  const int qb = nqb - 1 - blockIdx.y;
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
    mx = max_over_halves(mx);
    const float m_new = fmaxf(m_run, mx);      // finite from the first tile on (key 0 is visible)
    if (__any((m_new - m_run) * scale2 > kSlack)) {      // see kSlack
      const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
      l_run *= corr;
#pragma unroll
      for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] *= corr;
      m_run = m_new;
    }
    const float mneg = -m_run * scale2;
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
    l_run += lsum;
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


// ---------------------------------------------------------------------------------------
// Long chunks: 384 queries x one head per workgroup of twelve waves (32 queries each, three
// waves per SIMD: what hides the latencies here is other waves), K and V tiles of 64 keys
// copied global -> LDS by the buffer-load-to-LDS path into a ring of four stages (three tiles in
// flight, no staging registers, no address arithmetic per element), both stored row-major
// [key][dim].  The V^T fragments the second product needs are read with the LDS transpose
// read: in a group of 16 lanes, lane 4j + a supplies dims 4a .. 4a+3 of key j, and lane i
// receives dim i of keys 0 .. 3 -- so the 16 lanes read a 4-key x 16-dim patch and end up
// holding one dim each, in order.  16-byte chunks of a row are XOR-swizzled by the key so
// that neither the K row reads nor the V patch reads collide on LDS banks; the swizzle is
// applied on the global side of the copy (the LDS side of it is linear).
namespace dma {

#ifndef ECHOKV_LDS
#define ECHOKV_LDS __attribute__((address_space(3)))
#endif
using fused::rsrc_t;
typedef short short4_t __attribute__((ext_vector_type(4)));

// the first NCOPY waves issue the copies (a tile is 16 or 32 one-KB copies per operand)
constexpr int NST = 4, NCOPY = 8, NWAVES = 12, NTHREADS = 64 * NWAVES, BQ = 32 * NWAVES;
constexpr int kMinQueries = 1024;      // shorter chunks: split over the keys if the context is long, else the four-wave kernel
constexpr int kMaxSplits = 8;

template <int HD> struct Cfg {
  static constexpr int ROWB = HD * 2;                   // bytes per key row
  static constexpr int CH = HD / 8;                     // 16-byte chunks per row
  static constexpr int TILE = BKV * ROWB;               // bytes of one K (or V) tile
  static constexpr int STAGE = 2 * TILE;                // K tile then V tile
  static constexpr int NL = TILE / 1024 / NCOPY;        // 1 KB copies per copying wave, tile and operand
  static constexpr int ROWS_PER_COPY = 1024 / ROWB;     // 4 (HD = 128) or 8 (HD = 64)
  static constexpr int KSTEPS = HD / 16, CB = HD / 32;
  // chunk c of key row r is stored at chunk c ^ kswz(r) (K tile) / c ^ vswz(r) (V tile)
  __device__ static __forceinline__ int kswz(int r) { return CH == 16 ? (r & 15) : ((r ^ (r >> 3)) & 7); }
  __device__ static __forceinline__ int vswz(int r) { return CH == 16 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); }
};

template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));   // vmcnt(N)
  __builtin_amdgcn_s_waitcnt(0xC07F);                                   // lgkmcnt(0): own LDS reads done
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// What a lane needs to issue its share of a tile's global -> LDS copies: copy i of a copying
// wave fills tile rows (NL wave + i) * ROWS_PER_COPY + lane / CH; LDS chunk slot lane % CH of
// such a row receives global chunk slot ^ swizzle(row).  Copy i sits i * ROWS_PER_COPY rows
// below copy 0: same V swizzle; the K swizzle of d = 128 (row & 15, copy 0 in rows 0..3 mod 16)
// changes by 4 i mod 16 (d = 64 has one copy per wave and operand).
template <int HD> struct CopyPlan {
  rsrc_t rk, rv;
  int row0;                             // tile row of copy 0
  uint32_t kcol0, vcol0;                // byte offset of its (swizzled) source chunk in the row
  uint32_t ld2; int last, wave_u;
};
// Issue this wave's copies of key tile t into ring stage t % NST.  Rows past the last key
// repeat it: finite values, masked by causality.  (A device function of its own: the copy
// builtin is not accepted inside a kernel body by the host pass.)
// (TAG: every kernel instantiation uses a specialisation of its own.  The host pass cannot compile
// the copy builtin; it lets that pass for the first kernel that uses a specialisation and then
// refuses the same specialisation to a second one.)
template <int HD, int TAG>
__device__ __forceinline__ void dma_tile(char* smem, const CopyPlan<HD>& cp, int t) {
  using C = Cfg<HD>;
  static_assert(C::NL == 1 || (C::CH == 16 && C::ROWS_PER_COPY == 4), "swizzle relation between a wave's copies");
  if (cp.wave_u >= NCOPY) return;
  char* st = smem + (t & (NST - 1)) * C::STAGE;
  const int kv0 = t * BKV;
#pragma unroll
  for (int i = 0; i < C::NL; ++i) {
    const uint32_t ro = __umul24((uint32_t)min(kv0 + cp.row0 + i * C::ROWS_PER_COPY, cp.last), cp.ld2);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(cp.rk, (ECHOKV_LDS void*)(st + (C::NL * cp.wave_u + i) * 1024), 16,
                                             ro + (cp.kcol0 ^ (uint32_t)(((i * 4) & 15) << 4)), 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(cp.rv, (ECHOKV_LDS void*)(st + C::TILE + (C::NL * cp.wave_u + i) * 1024), 16,
                                             ro + cp.vcol0, 0, 0, 0);
  }
}

typedef short short8_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(ECHOKV_LDS const char*)p;
}
// One k-step's V^T fragments: per 32-dim block, keys k0 .. k0+3 (lo) and k0+8 .. k0+11 (hi).
struct VFrag { short4_t lo[4], hi[4]; };
// The LDS transpose reads are written as instructions: in builtin form the compiler orders
// them behind every outstanding global -> LDS copy (s_waitcnt vmcnt(0)), which would drain the
// ring once per tile.  issue_v requests the fragments of k-step TS; wait_v<N> waits until at
// most N reads requested after them are outstanding, its operands tie it to the registers it
// guards.  voff0: this lane's byte offset inside a V tile for k-step 0 and 32-dim block 0; block
// cb is at voff0 ^ (cb << 6) (the swizzle only touches the two chunk-index bits that cb occupies).
#define ECHOKV_TR(dst, adr, off) "ds_read_b64_tr_b16 " dst ", " adr " offset:" off "\n"
template <int HD, int TS>
__device__ __forceinline__ void issue_v(VFrag& f, uint32_t sv, uint32_t voff0) {
  constexpr int LO = 16 * TS * Cfg<HD>::ROWB, HI = (16 * TS + 8) * Cfg<HD>::ROWB;
  if constexpr (Cfg<HD>::CB == 4) {
    asm volatile(ECHOKV_TR("%0", "%8", "%12") ECHOKV_TR("%4", "%8", "%13")
                 ECHOKV_TR("%1", "%9", "%12") ECHOKV_TR("%5", "%9", "%13")
                 ECHOKV_TR("%2", "%10", "%12") ECHOKV_TR("%6", "%10", "%13")
                 ECHOKV_TR("%3", "%11", "%12") ECHOKV_TR("%7", "%11", "%13")
                 : "=&v"(f.lo[0]), "=&v"(f.lo[1]), "=&v"(f.lo[2]), "=&v"(f.lo[3]),
                   "=&v"(f.hi[0]), "=&v"(f.hi[1]), "=&v"(f.hi[2]), "=&v"(f.hi[3])
                 : "v"(sv + voff0), "v"(sv + (voff0 ^ 64u)), "v"(sv + (voff0 ^ 128u)), "v"(sv + (voff0 ^ 192u)), "n"(LO), "n"(HI));
  } else {
    asm volatile(ECHOKV_TR("%0", "%4", "%6") ECHOKV_TR("%2", "%4", "%7")
                 ECHOKV_TR("%1", "%5", "%6") ECHOKV_TR("%3", "%5", "%7")
                 : "=&v"(f.lo[0]), "=&v"(f.lo[1]), "=&v"(f.hi[0]), "=&v"(f.hi[1])
                 : "v"(sv + voff0), "v"(sv + (voff0 ^ 64u)), "n"(LO), "n"(HI));
  }
}
template <int N, int CB>
__device__ __forceinline__ void wait_v(VFrag& f) {
  if constexpr (CB == 4)
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(f.lo[0]), "+v"(f.lo[1]), "+v"(f.lo[2]), "+v"(f.lo[3]),
                   "+v"(f.hi[0]), "+v"(f.hi[1]), "+v"(f.hi[2]), "+v"(f.hi[3])
                 : "n"(N));
  else
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(f.lo[0]), "+v"(f.lo[1]), "+v"(f.hi[0]), "+v"(f.hi[1]) : "n"(N));
}

template <int HD, bool SPLIT>
__global__ __launch_bounds__(NTHREADS) void prefill_attn_dma_kernel(Args a) {
  using C = Cfg<HD>;
  extern __shared__ __attribute__((aligned(1024))) char smem[];      // NST stages of [K tile | V tile]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int lr = lane & 31, lh = lane >> 5;
  const int h = blockIdx.x;                       // grid = (heads, query blocks), longest blocks of all heads first
  // Query blocks are counted from the END of the chunk: block y covers queries
  // [T_q - (y + 1) BQ, T_q - y BQ).  If T_q is not a multiple of BQ the block that is only partly
  // filled is then the first (shortest, cheapest) one and not the last (longest) one; its queries
  // below 0 repeat query 0 and are not written back.
  const int i0 = a.T_q - ((int)blockIdx.y + 1) * BQ;
  const int Ltot = a.q_pos0 + a.T_q;
  const int kvh = h / a.G;
  const bf16_t* kbase; const bf16_t* vbase; uint32_t ld2;
  if (kvh < a.n_ret_heads) { kbase = a.k_ret + kvh * HD; vbase = a.v_ret + kvh * HD; ld2 = (uint32_t)a.m * 2; }
  else { const int c = (kvh - a.n_ret_heads) * HD; kbase = a.k_hat + c; vbase = a.v_hat + c; ld2 = (uint32_t)a.d_out * 2; }

  CopyPlan<HD> cp;
  cp.row0 = C::NL * wave_u * C::ROWS_PER_COPY + lane / C::CH;
  cp.kcol0 = (uint32_t)(((lane % C::CH) ^ C::kswz(cp.row0)) * 16);
  cp.vcol0 = (uint32_t)(((lane % C::CH) ^ C::vswz(cp.row0)) * 16);
  cp.rk = fused::make_rsrc(kbase); cp.rv = fused::make_rsrc(vbase);
  cp.ld2 = ld2; cp.last = Ltot - 1; cp.wave_u = wave_u;

  // ---- this lane's query (clamped; clamped duplicates are not written back)
  const int qi = i0 + wave_u * 32 + lr;
  const int qic = max(qi, 0);                     // (qi < T_q always: blocks end at T_q - y BQ)
  bf16x8_t qf[C::KSTEPS];
  {
    const bf16_t* qp = a.q + ((int64_t)qic * a.H_q + h) * HD + lh * 8;
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk) qf[kk] = *reinterpret_cast<const bf16x8_t*>(qp + kk * 16);
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the ring's load counting starts from zero
  asm volatile("" ::: "memory");
  floatx16_t oacc[C::CB];
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float scale2 = a.scale * 1.44269504088896340736f;    // softmax in base 2
  const int qpos_min = a.q_pos0 + max(i0 + wave_u * 32, 0);
  const int qpos_max = a.q_pos0 + max(i0 + wave_u * 32 + 31, 0);
  const int kv_end = min(Ltot, a.q_pos0 + i0 + BQ);   // keys any query of the block sees (i0 + BQ <= T_q)
  const int ntiles_blk = (kv_end + BKV - 1) / BKV;
  // SPLIT: this workgroup's share [t_first, ntiles) of the block's key tiles
  int t_first = 0, ntiles = ntiles_blk;
  if constexpr (SPLIT) {
    const int per = (ntiles_blk + a.kv_splits - 1) / a.kv_splits;
    t_first = min((int)blockIdx.z * per, ntiles_blk);
    ntiles = min(ntiles_blk, t_first + per);
  }

  // ---- fragment addresses inside a stage
  // K: row mb*32 + lr, chunk (2 kk + lh) ^ kswz(row)
  // V: transpose read of the patch keys k0 + s/4, dims cb*32 + 16*(blk%2) + 4*(s%4) .. +3, with
  //    s = lane % 16, blk = lane / 16 (blk / 2 = lh): this lane then holds dim cb*32 + lane % 32
  const int s16 = lane & 15, blk2 = (lane >> 4) & 1;
  const int vkey = 4 * lh + (s16 >> 2);                        // + 16 ts (+ 8 for the second half)
  const int vch = 2 * blk2 + ((s16 & 3) >> 1);                 // + 4 cb, before the swizzle
  const uint32_t vbyte = (uint32_t)((s16 & 1) * 8);
  const uint32_t voff = (uint32_t)(vkey * C::ROWB + ((vch ^ C::vswz(vkey)) << 4)) + vbyte;   // see issue_v
  uint32_t koff[2];                      // K fragment of k-step 0: row mb*32 + lr, chunk lh ^ swizzle(row)
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) koff[mb] = (uint32_t)((mb * 32 + lr) * C::ROWB + ((lh ^ C::kswz(mb * 32 + lr)) << 4));

  // Two loops (tiles that reach a query of this wave, then tiles wholly past them where the
  // wave only keeps copying and meeting the others) instead of a skip inside one: no values
  // to merge between the paths.
  const int nact = min(ntiles, qpos_max / BKV + 1);
  dma_tile<HD, SPLIT ? 1 : 0>(smem, cp, t_first); dma_tile<HD, SPLIT ? 1 : 0>(smem, cp, t_first + 1); dma_tile<HD, SPLIT ? 1 : 0>(smem, cp, t_first + 2);
  int t = t_first;
  for (; t < nact; ++t) {
    wait_loads_and_barrier<2 * 2 * C::NL>();     // tile t has landed for every wave; stage (t-1)%NST is free
    dma_tile<HD, SPLIT ? 1 : 0>(smem, cp, t + 3);
    const int kv0 = t * BKV;
    const char* sk = smem + (t & (NST - 1)) * C::STAGE;
    const char* sv = sk + C::TILE;
    // ---- S^T = K Q^T
    const uint32_t svu = lds_addr(sv);
    floatx16_t sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[mb][r] = 0.f;
    // chunk (2 kk + lh) ^ swizzle of the lane's row is the chunk of k-step 0 with kk << 1 XOR-ed
    // in: one address register per key block serves all k-steps
#pragma unroll
    for (int kk = 0; kk < C::KSTEPS; ++kk)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sk + (koff[mb] ^ (uint32_t)(kk << 5)));
        sacc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[mb], 0, 0, 0);
      }
    // ---- online softmax, lane-local (keys: mb*32 + 8*(r/4) + 4*lh + r%4), base 2, scale folded in
    if (kv0 + BKV - 1 > qpos_min) {   // rare (diagonal tiles): the lane's query position is worked out afresh
      const int ln = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
      const int qp = a.q_pos0 + max(i0 + wave_u * 32 + (ln & 31), 0);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + mb * 32 + (r >> 2) * 8 + (ln >> 5) * 4 + (r & 3);
          if (key > qp) sacc[mb][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mb][r]);
    mx = max_over_halves(mx);
    // !SPLIT: finite from the first tile on (key 0 is visible to every query).  SPLIT: a share
    // that starts on the diagonal can leave a query with no visible key yet (-inf): its factor
    // is 1 and its probabilities are exp2(-inf + 0) = 0
    const float m_new = fmaxf(m_run, mx);
    if (__any((m_new - m_run) * scale2 > kSlack)) {      // see kSlack
      float corr = __builtin_amdgcn_exp2f((m_run - m_new) * scale2);
      if constexpr (SPLIT) corr = (m_new == -INFINITY) ? 1.f : corr;
      l_run *= corr;
#pragma unroll
      for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] *= corr;
      m_run = m_new;
    }
    float mneg = -m_run * scale2;
    if constexpr (SPLIT) mneg = (m_run == -INFINITY) ? 0.f : mneg;
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
    l_run += lsum;
    // ---- O^T += V^T P^T : k-step ts, element e of lane half lh <-> key 16 ts + 4 lh + (e < 4 ? e : e + 4).
    //      The transpose reads are issued by hand one k-step ahead of the MFMAs that use them.
    constexpr int V = 2 * C::CB;         // reads per k-step
    VFrag va, vb;
    auto pv = [&](int ts, const VFrag& v) {
#pragma unroll
      for (int cb = 0; cb < C::CB; ++cb) {
        const short8_t vv = __builtin_shufflevector(v.lo[cb], v.hi[cb], 0, 1, 2, 3, 4, 5, 6, 7);
        oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, vv), pf[ts], oacc[cb], 0, 0, 0);
      }
    };
    // two buffers: the fragments of a k-step are requested before the MFMAs of the one before it
    issue_v<HD, 0>(va, svu, voff);
    issue_v<HD, 1>(vb, svu, voff);
    wait_v<V, C::CB>(va); pv(0, va);
    issue_v<HD, 2>(va, svu, voff);
    wait_v<V, C::CB>(vb); pv(1, vb);
    issue_v<HD, 3>(vb, svu, voff);
    wait_v<V, C::CB>(va); pv(2, va);
    wait_v<0, C::CB>(vb); pv(3, vb);
  }
  for (; t < ntiles; ++t) {
    wait_loads_and_barrier<2 * 2 * C::NL>();
    dma_tile<HD, SPLIT ? 1 : 0>(smem, cp, t + 3);
  }
  wait_loads_and_barrier<0>();         // the ring's last copies have landed before the workgroup ends
  // ---- finish: this lane holds query qi, head dims cb*32 + 8*(r/4) + 4*lh + r%4
  //      (The lane index is read afresh so that nothing of the set-up stays in registers over the loop.)
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  const int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int lh_e = lane_e >> 5;
  const int qi_e = i0 + wave_u * 32 + (lane_e & 31);
  if (qi_e < 0) return;
  if constexpr (SPLIT) {        // unnormalised partial of this share: (max, sum, O)
    const int64_t pr = ((int64_t)qi_e * a.H_q + h) * a.kv_splits + blockIdx.z;
#pragma unroll
    for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *reinterpret_cast<float4*>(a.part_o + pr * HD + cb * 32 + r4 * 8 + lh_e * 4) =
            make_float4(oacc[cb][r4 * 4], oacc[cb][r4 * 4 + 1], oacc[cb][r4 * 4 + 2], oacc[cb][r4 * 4 + 3]);
    if (lh_e == 0) { a.part_ml[pr * 2] = m_run * scale2; a.part_ml[pr * 2 + 1] = l_tot; }
    return;
  }
  const float inv = 1.0f / l_tot;
  const int64_t ob = ((int64_t)qi_e * a.H_q + h) * HD;
#pragma unroll
  for (int cb = 0; cb < C::CB; ++cb)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      const int c = cb * 32 + r4 * 8 + lh_e * 4;
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
  if (a.lse && lh_e == 0)
    a.lse[(int64_t)qi_e * a.H_q + h] = (m_run * scale2 + __log2f(l_tot)) * 0.69314718055994530942f;
}

// Joins the key shares of a split launch: exact re-association of the softmax-weighted sums.
// One thread per (query, head, 4 head dims).
template <typename TO>
__global__ __launch_bounds__(256) void prefill_merge_kernel(Args a, int HD) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int q4 = HD / 4;
  const int64_t row = idx / q4;                    // query * H_q + head
  if (row >= (int64_t)a.T_q * a.H_q) return;
  const int c = (int)(idx % q4) * 4;
  const float* ml = a.part_ml + row * a.kv_splits * 2;
  float M = -INFINITY;
  for (int s = 0; s < a.kv_splits; ++s) M = fmaxf(M, ml[2 * s]);     // share 0 holds key 0: finite
  float l = 0.f;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < a.kv_splits; ++s) {
    const float ms = ml[2 * s];
    const float w = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - M);
    l = fmaf(w, ml[2 * s + 1], l);
    const float4 v = *reinterpret_cast<const float4*>(a.part_o + (row * a.kv_splits + s) * HD + c);
    o.x = fmaf(w, v.x, o.x); o.y = fmaf(w, v.y, o.y); o.z = fmaf(w, v.z, o.z); o.w = fmaf(w, v.w, o.w);
  }
  const float inv = 1.0f / l;
  TO* out = reinterpret_cast<TO*>(a.out) + row * HD + c;
  if constexpr (sizeof(TO) == 2) {
    uint2 w2;
    w2.x = (uint32_t)f32_to_bf16(o.x * inv) | ((uint32_t)f32_to_bf16(o.y * inv) << 16);
    w2.y = (uint32_t)f32_to_bf16(o.z * inv) | ((uint32_t)f32_to_bf16(o.w * inv) << 16);
    *reinterpret_cast<uint2*>(out) = w2;
  } else {
    *reinterpret_cast<float4*>(out) = make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
  }
  if (a.lse && c == 0) a.lse[row] = (M + __log2f(l)) * 0.69314718055994530942f;
}

template <int HD, bool SPLIT>
inline int launch(dim3 grid, dim3 blk, hipStream_t st, const Args& a) {
  constexpr int lds = NST * Cfg<HD>::STAGE;          // 128 KB (d = 128) or 64 KB of dynamic LDS
  void (*fn)(Args) = prefill_attn_dma_kernel<HD, SPLIT>;
  static bool allowed[64] = {};                      // per device: the attribute is set once
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 7;
  if (!allowed[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
      return 7;
    allowed[dev] = true;
  }
  hipLaunchKernelGGL(fn, grid, blk, lds, st, a);
  return hipGetLastError() != hipSuccess ? 7 : 0;
}

}  // namespace dma

}  // namespace prefill

// Rotary embedding of key rows ahead of the prefill attention kernels (Sec. "Network
// Architecture": caches hold pre-rotation keys): row j of src [rows, n_heads * d] (pitch
// ld_src) is rotated to position j, feature i of a head pairing with i + d/2, and written
// to dst (pitch ld_dst; dst may be src).  One thread per 8 + 8 paired features.
struct RopeRowsArgs {
  const bf16_t* src; bf16_t* dst;
  int64_t ld_src, ld_dst;
  int32_t n_heads, d, rows;
  const float* cos; const float* sin;      // [>= rows, d / 2]
};
__global__ __launch_bounds__(256) void rope_rows_kernel(RopeRowsArgs a) {
  const int cpr = a.d / 16;                               // threads per head
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_row = (int64_t)a.n_heads * cpr;
  if (idx >= per_row * a.rows) return;
  const int row = (int)(idx / per_row);
  const int rem = (int)(idx % per_row), head = rem / cpr, c = rem % cpr;
  const int half = a.d / 2;
  const bf16_t* sp = a.src + (int64_t)row * a.ld_src + head * a.d + c * 8;
  const fused::u32x4_t xa = *reinterpret_cast<const fused::u32x4_t*>(sp);
  const fused::u32x4_t xb = *reinterpret_cast<const fused::u32x4_t*>(sp + half);
  const float* cr = a.cos + (int64_t)row * half + c * 8;
  const float* sr = a.sin + (int64_t)row * half + c * 8;
  fused::u32x4_t ya, yb;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    uint32_t oa = 0, ob = 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float fa = __uint_as_float(((xa[w] >> (16 * e)) & 0xffffu) << 16);
      const float fb = __uint_as_float(((xb[w] >> (16 * e)) & 0xffffu) << 16);
      const float cs = cr[2 * w + e], sn = sr[2 * w + e];
      oa |= (uint32_t)f32_to_bf16(fa * cs - fb * sn) << (16 * e);
      ob |= (uint32_t)f32_to_bf16(fb * cs + fa * sn) << (16 * e);
    }
    ya[w] = oa; yb[w] = ob;
  }
  bf16_t* dp = a.dst + (int64_t)row * a.ld_dst + head * a.d + c * 8;
  *reinterpret_cast<fused::u32x4_t*>(dp) = ya;
  *reinterpret_cast<fused::u32x4_t*>(dp + half) = yb;
}
inline int launch_rope_rows(const bf16_t* src, int64_t ld_src, bf16_t* dst, int64_t ld_dst, int n_heads,
                            int d, int rows, const float* cos, const float* sin, hipStream_t st) {
  if (n_heads <= 0 || rows <= 0) return 0;
  RopeRowsArgs a;
  a.src = src; a.dst = dst; a.ld_src = ld_src; a.ld_dst = ld_dst; a.n_heads = n_heads; a.d = d;
  a.rows = rows; a.cos = cos; a.sin = sin;
  const int64_t n = (int64_t)rows * n_heads * (d / 16);
  hipLaunchKernelGGL(rope_rows_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, a);
  return hipGetLastError() != hipSuccess ? 7 : 0;
}

template <typename T> inline bool prefill_mfma_supported(int d) {
  return sizeof(T) == 2 && (d == 64 || d == 128);
}

// Key shares for a chunk of T_q queries over Ltot cached tokens (1 = no split).  Chunks of
// kMinQueries queries and more fill the chip by themselves.  A shorter chunk has at most three query
// blocks per head; with a long context in front of it each (head, block) is cut into shares of at
// least 8 key tiles until about three workgroups per compute unit exist.
inline int prefill_kv_splits(int T_q, int64_t Ltot, int H_q) {
  if (T_q >= prefill::dma::kMinQueries) return 1;
  const int wgs = (T_q + prefill::dma::BQ - 1) / prefill::dma::BQ * H_q;
  const int64_t tiles = (Ltot + prefill::BKV - 1) / prefill::BKV;
  int S = (int)std::min<int64_t>(prefill::dma::kMaxSplits, tiles / 8);
  S = std::min(S, (768 + wgs - 1) / wgs);
  return std::max(S, 1);
}
// fp32 words the partials of such a launch take: (d + 2) per (query, head, share)
inline size_t prefill_split_floats(int T_q, int64_t Ltot, int H_q, int d) {
  const int S = prefill_kv_splits(T_q, Ltot, H_q);
  return S > 1 ? (size_t)T_q * H_q * S * (d + 2) : 0;
}

// k_ret / v_ret: retained cache at the sequence's first row (stride m);
// k_hat / v_hat: predicted dims of tokens 0 .. q_pos0+T_q-1 (stride d_out).
template <typename T>
inline int launch_prefill_mfma(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                               float scale, bool out_bf16,
                               const T* k_ret, const T* v_ret, const T* k_hat, const T* v_hat,
                               const T* q, int T_q, int q_pos0, void* out, float* lse,
                               hipStream_t st, float* part_o = nullptr, float* part_ml = nullptr) {
  if constexpr (sizeof(T) != 2) {
    return 6;
  } else {
    prefill::Args a;
    a.k_ret = k_ret; a.v_ret = v_ret; a.k_hat = k_hat; a.v_hat = v_hat; a.q = q;
    a.out = out; a.lse = lse;
    a.H_q = H_q; a.G = H_q / H_kv; a.m = m; a.d_out = d_out; a.n_ret_heads = n_ret_heads;
    a.T_q = T_q; a.q_pos0 = q_pos0; a.out_bf16 = out_bf16 ? 1 : 0; a.scale = scale;
    a.kv_splits = 1; a.part_o = nullptr; a.part_ml = nullptr;
    // long chunks take the twelve-wave kernel with the LDS ring (its 32-bit row offsets must fit);
    // so do short chunks in front of a long context, split over the keys so that the grid still
    // fills the chip
    const int64_t span = (int64_t)(q_pos0 + T_q) * (m > d_out ? m : d_out) * 2;
    const int S = span < (int64_t)1 << 31 ? prefill_kv_splits(T_q, q_pos0 + T_q, H_q) : 1;
    if (S > 1) {
      if (!part_o || !part_ml) return 5;
      a.kv_splits = S; a.part_o = part_o; a.part_ml = part_ml;
      const dim3 grid(H_q, (T_q + prefill::dma::BQ - 1) / prefill::dma::BQ, S), blk(prefill::dma::NTHREADS);
      int rc = d == 128 ? prefill::dma::launch<128, true>(grid, blk, st, a) : prefill::dma::launch<64, true>(grid, blk, st, a);
      if (rc) return rc;
      const unsigned mb = (unsigned)(((int64_t)T_q * H_q * (d / 4) + 255) / 256);
      if (out_bf16) hipLaunchKernelGGL((prefill::dma::prefill_merge_kernel<bf16_t>), dim3(mb), dim3(256), 0, st, a, d);
      else hipLaunchKernelGGL((prefill::dma::prefill_merge_kernel<float>), dim3(mb), dim3(256), 0, st, a, d);
      return hipGetLastError() != hipSuccess ? 7 : 0;
    }
    if (T_q >= prefill::dma::kMinQueries && span < (int64_t)1 << 31) {
      const dim3 grid(H_q, (T_q + prefill::dma::BQ - 1) / prefill::dma::BQ), blk(prefill::dma::NTHREADS);
      return d == 128 ? prefill::dma::launch<128, false>(grid, blk, st, a) : prefill::dma::launch<64, false>(grid, blk, st, a);
    }
    dim3 grid(H_q, (T_q + prefill::BQ - 1) / prefill::BQ);
    if (d == 128) hipLaunchKernelGGL((prefill::prefill_attn_kernel<128>), grid, dim3(prefill::NTHREADS), 0, st, a);
    else hipLaunchKernelGGL((prefill::prefill_attn_kernel<64>), grid, dim3(prefill::NTHREADS), 0, st, a);
    if (hipGetLastError() != hipSuccess) return 7;
    return 0;
  }
}

}  // namespace echokv
