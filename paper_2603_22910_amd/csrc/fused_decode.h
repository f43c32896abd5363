// Fused reconstruct-then-attend decode kernel for gfx950 (bf16 MFMA), and the
// stand-alone predictor product that shares its main loop.
//
// One workgroup owns a tile of 256 cached tokens x 256 predicted columns
// (two heads of 128, or four of 64).  For that tile it
//   1. runs the predictor product for K (Eq. 3) on v_mfma_f32_32x32x16_bf16,
//      with W as the row operand so that each lane ends up holding whole
//      columns of K_hat^T for ONE token: the score q . k_hat_j (Eq. 7) is then a
//      sum over the lane's own accumulators plus one cross-half add;
//   2. takes the softmax numerators over each wave's 128 tokens (max, sum of
//      exponentials), leaving p_j in LDS;
//   3. runs the predictor product for V with X as the row operand, so each
//      lane holds rows (tokens) of V_hat for one column and sum_j p_j v_hat_j
//      is again lane-local;
//   4. writes one split-K partial (max, sum, unnormalised o) per wave and head.
// K_hat and V_hat live only in accumulator registers: they never reach LDS or HBM.
//
// The predictor input row [anchor ; retained] (Eq. 3) is never materialised
// either: the k-loop walks the anchor cache for the first D input dims and
// the target's retained cache for the last m.
#pragma once
#include "common.h"

namespace echokv {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx16_t __attribute__((ext_vector_type(16)));

namespace fused {

constexpr int BM = 256;      // tokens per workgroup tile
constexpr int BN = 256;      // predicted columns per workgroup tile
constexpr int BK = 64;       // input dims per pipeline stage
constexpr int NTHREADS = 256;
constexpr int WM = 128, WN = 128;   // per-wave tile (2 x 2 waves)
constexpr int MAXPAIR = 8;   // (head in wave tile, query head in group) pairs per wave

struct Args {
  const bf16_t* xa[2];   // anchor cache K, V      [pool, D]
  const bf16_t* xr[2];   // retained cache K, V    [pool, m]
  const bf16_t* w[2];    // W_K, W_V               [D + m, d_out]
  const bf16_t* q;       // [nseq, H_q, d]
  float* part_o;         // [slots, H_q, d]
  float* part_ml;        // [slots, H_q, 2]
  bf16_t* out[2];        // store kernel only: K_hat / V_hat destination
  int64_t ldo;           // store kernel: row stride (elements)
  int32_t col0;          // store kernel: first column
  int32_t D, m, d_out, H_q, G, n_ret_heads;
  float scale;
  int32_t n_col_tiles, n_tiles;   // column tiles; token tiles * column tiles
  // paper-faithful extras (null / zero: off): rotary tables [positions, d/2] applied to the rebuilt
  // keys by token position; tokens held by the uncompressed window are masked out here
  const float* rope_cos; const float* rope_sin;
  int32_t n_sink, n_recent;
  float* s_out;          // score kernel only: S^T [H_q, s_ld], column = slot * 128 + token
  int64_t s_ld;
};

// LDS tile: [rows][64 k] bf16, a row is 8 chunks of 16 bytes; chunk c of row r
// lives at chunk slot c ^ swz(r), swz(r) = (r ^ (r >> 3)) & 7, which keeps the
// 16-byte fragment reads of 16 consecutive rows, the row-contiguous X writes
// and the column-strided W writes all spread over the banks.  All addresses a
// thread ever needs are a handful of per-thread bases plus compile-time
// offsets; they are worked out once (struct Addr) so that the main loop
// carries no address arithmetic.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// LDS state of the attention epilogues (shared by the bf16 and fp32 kernels)
struct EpiSmem {
  float q[BN * MAXPAIR];               // [(head in tile * G + g)][d], pre-scaled
  float p[4][MAXPAIR][128];            // per wave and pair: softmax numerators of its 128 tokens
  float ml[4][MAXPAIR][2];             // per wave and pair: max and sum
};
struct Smem {
  char x[2][BM * BK * 2];
  char w[2][BN * BK * 2];
  EpiSmem e;
};
constexpr int kStageBytes = BM * BK * 2;          // one stage of x (same for w)
constexpr int kWBase = 2 * kStageBytes;           // offset of Smem::w from Smem::x

struct Addr {
  // fragment reads: row = wave base + 32*i + lr, chunk = 2*kk + lh.
  // byte offset = fr[kk][i & 1] + (i >> 1) * 8192 (+ operand / stage base)
  uint32_t frx[4][2], frw[4][2];
  // X writes: row = 32*i + tid/8, chunk = tid & 7: wx[i & 1] + (i >> 1) * 8192
  uint32_t wx[2];
  // W writes: row = 8*(tid & 31) + j, chunk = tid >> 5: ww[j]
  uint32_t ww[8];
};

__device__ __forceinline__ void make_addr(Addr& ad, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1;
  const int lr = lane & 31, lh = lane >> 5;
  const int flr = (lr ^ (lr >> 3)) & 7;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
#pragma unroll
    for (int ip = 0; ip < 2; ++ip) {
      const uint32_t o = (uint32_t)((ip * 32 + lr) * 128 + (((kk * 2 + lh) ^ flr ^ (ip << 2)) << 4));
      ad.frx[kk][ip] = o + wt * (WM * 128);
      ad.frw[kk][ip] = o + wc * (WN * 128) + kWBase;
    }
  const int r0 = tid >> 3, c = tid & 7;
  const int f0 = (r0 ^ (r0 >> 3)) & 7;
#pragma unroll
  for (int ip = 0; ip < 2; ++ip)
    ad.wx[ip] = (uint32_t)((ip * 32 + r0) * 128 + ((c ^ f0 ^ (ip << 2)) << 4));
  const int nb = tid & 31, kb = tid >> 5;
#pragma unroll
  for (int j = 0; j < 8; ++j)
    ad.ww[j] = (uint32_t)((nb * 8 + j) * 128 + (((kb ^ j ^ nb) & 7) << 4)) + kWBase;
}

// global -> registers for one k-tile.  X: 8 x 16B per thread; W: an 8x8 block.
struct Stage {
  u32x4_t x[8];
  u32x4_t w[8];
};

// Per-thread global offsets, fixed for a pass.
struct GOff {
  uint32_t r0;        // tile row of X load 0 (load i reads row min(r0 + 32 i, last))
  uint32_t last;      // last valid row of the tile
  uint32_t xcol;      // byte offset of this thread's 16-byte chunk in a 128-byte k-slab
  uint32_t w0;        // byte offset of this thread's W block inside a k-tile of W
  uint32_t wlast;     // packed weights: last valid row (output column) of the W^T tile
};

__device__ __forceinline__ void make_goff(GOff& g, int tid, int last, int d_out, int nclamp) {
  g.r0 = (uint32_t)(tid >> 3);
  g.last = (uint32_t)last;
  g.xcol = (uint32_t)(tid & 7) * 16;
  const int nb = tid & 31, kb = tid >> 5;
  // column blocks past d_out are clamped onto the last valid block: the heads
  // they would feed are skipped in the epilogue, they only need to be readable
  g.w0 = (uint32_t)(kb * 8) * (uint32_t)(d_out * 2) + (uint32_t)min(nb * 8, nclamp) * 2;
  g.wlast = (uint32_t)min(BN - 1, nclamp + 7);
}

// Global loads go through raw buffer instructions: a 128-bit resource
// (uniform base) + a 32-bit per-thread byte offset + a uniform byte offset, so
// no 64-bit address arithmetic is spent per load.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
  // raw buffer, no stride, byte-granular range check far beyond any offset used here
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
struct Src {
  rsrc_t xa, xr, w;    // anchor tile rows, retained tile rows, W + n0
};

// Issue the global loads of k-tile `kn` (8 for X, 8 for W).
__device__ __forceinline__ void fetch_x(Stage& s, const GOff& g, const Src& src, int D, int m,
                                        int nka, int kn) {
  // anchor dims first, then retained dims (Eq. 3); uniform selects, no branch
  const bool anchor = kn < nka;
  const uint32_t ld2 = (uint32_t)(anchor ? D : m) * 2;
  const int soff = (anchor ? kn : kn - nka) * (BK * 2);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t voff = __umul24(min(g.r0 + 32u * i, g.last), ld2) + g.xcol;   // row < 256, ld2 < 2^24
    s.x[i] = anchor ? __builtin_amdgcn_raw_buffer_load_b128(src.xa, voff, soff, 0)
                    : __builtin_amdgcn_raw_buffer_load_b128(src.xr, voff, soff, 0);
  }
}
// PACKED: the weights were transposed once to [d_out, d_in] (echokv_pack_weights),
// so a W^T tile is fetched exactly like an X tile: rows = output columns, 64
// input dims contiguous.  Otherwise W is [d_in, d_out] and every thread
// fetches an 8 (k) x 8 (n) block that store_w transposes on the way to LDS.
template <bool PACKED>
__device__ __forceinline__ void fetch_w(Stage& s, const GOff& g, const Src& src, int d_in,
                                        int d_out, int kn) {
  if constexpr (PACKED) {
    const uint32_t ld2 = (uint32_t)d_in * 2;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t voff = __umul24(min(g.r0 + 32u * i, g.wlast), ld2) + g.xcol;
      s.w[i] = __builtin_amdgcn_raw_buffer_load_b128(src.w, voff, kn * (BK * 2), 0);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      s.w[i] = __builtin_amdgcn_raw_buffer_load_b128(src.w, g.w0, (kn * BK + i) * d_out * 2, 0);
  }
}
template <bool PACKED>
__device__ __forceinline__ void fetch_tile(Stage& s, const GOff& g, const Src& src, int D, int m,
                                           int d_out, int nka, int kn) {
  fetch_x(s, g, src, D, m, nka, kn);
  fetch_w<PACKED>(s, g, src, D + m, d_out, kn);
}

__device__ __forceinline__ void store_x(const Stage& s, char* smem, int stage, const Addr& ad) {
#pragma unroll
  for (int i = 0; i < 8; ++i)
    *reinterpret_cast<u32x4_t*>(smem + ad.wx[i & 1] + (i >> 1) * 8192 + stage * kStageBytes) = s.x[i];
}

// 8x8 transpose of 16-bit elements held as 8 rows (k) of 4 dwords (8 n), then
// 8 row writes: LDS row n (a W column) gets its 8 consecutive k values.
// One byte-permute per output dword.
template <bool PACKED>
__device__ __forceinline__ void store_w(const Stage& s, char* smem, int stage, const Addr& ad) {
  if constexpr (PACKED) {      // rows arrive k-contiguous: same placement as an X tile
#pragma unroll
    for (int i = 0; i < 8; ++i)
      *reinterpret_cast<u32x4_t*>(smem + ad.wx[i & 1] + (i >> 1) * 8192 + kWBase + stage * kStageBytes) = s.w[i];
    return;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    u32x4_t o;
#pragma unroll
    for (int pq = 0; pq < 4; ++pq) {
      const uint32_t a = s.w[2 * pq][j >> 1], b = s.w[2 * pq + 1][j >> 1];
      o[pq] = __builtin_amdgcn_perm(b, a, (j & 1) ? 0x07060302u : 0x05040100u);
    }
    *reinterpret_cast<u32x4_t*>(smem + ad.ww[j] + stage * kStageBytes) = o;
  }
}

struct Frags {
  bf16x8_t x[4], w[4];
};

__device__ __forceinline__ void load_frags(Frags& f, const char* smem, int stage, int kk,
                                           const Addr& ad) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f.x[i] = *reinterpret_cast<const bf16x8_t*>(smem + ad.frx[kk][i & 1] + (i >> 1) * 8192 + stage * kStageBytes);
    f.w[i] = *reinterpret_cast<const bf16x8_t*>(smem + ad.frw[kk][i & 1] + (i >> 1) * 8192 + stage * kStageBytes);
  }
}

// 16 MFMAs of one k-step.  SWAP: accumulator block [ci][ji] = W^T x X^T (rows =
// output columns, lanes = tokens); otherwise [ji][ci] = X x W (rows = tokens,
// lanes = output columns).
template <bool SWAP>
__device__ __forceinline__ void mma16(floatx16_t (&acc)[4][4], const Frags& f) {
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      if constexpr (SWAP)
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.w[a], f.x[b], acc[a][b], 0, 0, 0);
      else
        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.x[a], f.w[b], acc[a][b], 0, 0, 0);
    }
}

// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
constexpr int SG_VALU = 0x2, SG_MFMA = 0x8, SG_VMEM_RD = 0x20, SG_DS_RD = 0x100, SG_DS_WR = 0x200;

// One k-tile (64 input dims) of the pipeline, for the LDS stage STAGE.  Every
// step issues 16 MFMAs, the 8 fragment reads of the next step and 8 memory
// operations of the prefetch, dealt out between the MFMAs so that neither the
// matrix pipe nor the memory queues see a burst:
//   step 0: k-step 0 | X part of tile kt+1: registers -> LDS (other stage)
//   step 1: k-step 1 | W part of tile kt+1: 8x8 transposes, registers -> LDS
//   step 2: k-step 2 | X part of tile kt+3: global -> registers ; barrier
//   step 3: k-step 3 | W part of tile kt+3: global -> registers ; first fragments of tile kt+1
// f0 holds the fragments of k-step 0 on entry and on exit.
template <bool SWAP, bool PACKED, int STAGE, bool STORE, bool FETCH>
__device__ __forceinline__ void k_tile(floatx16_t (&acc)[4][4], Frags& f0, Frags& f1, Stage& st,
                                       char* smem, const Addr& ad, const GOff& g, const Src& src,
                                       int D, int m, int d_out, int nka, int kfetch) {
  // ---- step 0.  LDS reads stay ahead of the LDS writes (the compiler must
  // assume they may alias), and the writes keep their program order.
  load_frags(f1, smem, STAGE, 1, ad);
  if constexpr (STORE) store_x(st, smem, STAGE ^ 1, ad);
  mma16<SWAP>(acc, f0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    SGB(SG_MFMA, 1);
    SGB(SG_DS_RD, 1);
  }
  if constexpr (STORE) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_WR, 1);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- step 1
  load_frags(f0, smem, STAGE, 2, ad);
  if constexpr (STORE) store_w<PACKED>(st, smem, STAGE ^ 1, ad);
  mma16<SWAP>(acc, f1);
  if constexpr (STORE && PACKED) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_RD, 1);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_WR, 1);
    }
  } else if constexpr (STORE) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_RD, 2);
      SGB(SG_VALU, 4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_WR, 1);
      SGB(SG_VALU, 4);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_WR, 1);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      SGB(SG_MFMA, 1);
      SGB(SG_DS_RD, 1);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- step 2
  load_frags(f1, smem, STAGE, 3, ad);
  if constexpr (FETCH) fetch_x(st, g, src, D, m, nka, kfetch);
  mma16<SWAP>(acc, f0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    SGB(SG_MFMA, 1);
    SGB(SG_DS_RD, 1);
    if constexpr (FETCH) {
      SGB(SG_VALU, 3);
      SGB(SG_MFMA, 1);
      SGB(SG_VMEM_RD, 1);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  // every wave has read all it needs from STAGE and (STORE) finished writing the
  // other stage; __syncthreads waits for this wave's LDS traffic first
  __syncthreads();
  // ---- step 3
  load_frags(f0, smem, STAGE ^ 1, 0, ad);
  if constexpr (FETCH) fetch_w<PACKED>(st, g, src, D + m, d_out, kfetch);
  mma16<SWAP>(acc, f1);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    SGB(SG_MFMA, 1);
    SGB(SG_DS_RD, 1);
    if constexpr (FETCH) {
      if constexpr (PACKED) SGB(SG_VALU, 3);
      SGB(SG_MFMA, 1);
      SGB(SG_VMEM_RD, 1);
    }
  }
  __builtin_amdgcn_sched_barrier(0);
}

// Full k-loop over d_in = D + m for one of the two products.  On return every
// wave is past its last LDS read of the stage buffers' final tile only after
// the caller's next barrier; the p / q / ml regions are never touched here.
//   xa_tile / xr_tile: first row of the token tile in the anchor / retained cache
//   last: index (in the tile) of the last valid row;  w_tile: W + n0
// What a pass needs to address its operands; rebuilt per pass (see gemm_pass).
struct PassIo {
  GOff g;
  Src src;
  int nk, nka, rot;
  // k-tiles are visited in a rotated order (tile (i + rot) mod nk at step i):
  // cache rows are a power of two bytes apart, so workgroups that walked the
  // input dims in the same order would all pull from one memory channel at a
  // time.  Indices past the end are clamped (a redundant, harmless reload) so
  // that every tile runs the same code.
  __device__ __forceinline__ int ktile(int i) const {
    const int t = min(i, nk - 1) + rot;
    return t >= nk ? t - nk : t;
  }
};

__device__ __forceinline__ void make_io(PassIo& io, const Args& a, const bf16_t* xa_tile,
                                        const bf16_t* xr_tile, const bf16_t* w_tile, int last,
                                        int nclamp, int tid_in, int rot) {
  // built from an opaque copy of the thread id: values that stayed live across
  // the register-hungry epilogues would be spilled and reloaded inside the main loop
  int tid = tid_in;
  asm volatile("" : "+v"(tid));
  make_goff(io.g, tid, last, a.d_out, nclamp);
  io.src.xa = make_rsrc(xa_tile); io.src.xr = make_rsrc(xr_tile); io.src.w = make_rsrc(w_tile);
  io.nk = (a.D + a.m) / BK; io.nka = a.D / BK; io.rot = rot;
}

// Issue the global loads of a pass's first k-tile.  Called before the
// previous pass's epilogue so that their latency hides behind it.
template <bool PACKED>
__device__ __forceinline__ void pass_prefetch(Stage& sa, const PassIo& io, const Args& a) {
  fetch_tile<PACKED>(sa, io.g, io.src, a.D, a.m, a.d_out, io.nka, io.ktile(0));
}

// Full k-loop over d_in = D + m for one of the two products; sa holds (or is
// about to receive) k-tile 0.
// Two register stages: k-tile t travels global -> sa (t even) / sb (t odd)
// -> LDS stage t & 1.  Tile t is fetched during tile t-3, written to LDS
// during tile t-1 and multiplied during tile t, so a global load has almost
// two tiles of MFMA time to land.
template <bool SWAP, bool PACKED>
__device__ __forceinline__ void gemm_pass(floatx16_t (&acc)[4][4], char* smem, const Args& a,
                                          const PassIo& io, Stage& sa, Stage& sb, int tid_in) {
  int tid = tid_in;
  asm volatile("" : "+v"(tid));
  Addr ad;
  make_addr(ad, tid);
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const int D = a.D, m = a.m, d_out = a.d_out;
  const int nk = io.nk, nka = io.nka;
  const GOff& g = io.g;
  const Src& src = io.src;
  Frags f0, f1;
  __syncthreads();     // the previous pass is done with the stage buffers
  fetch_tile<PACKED>(sb, g, src, D, m, d_out, nka, io.ktile(1));
  store_x(sa, smem, 0, ad);
  store_w<PACKED>(sa, smem, 0, ad);
  fetch_tile<PACKED>(sa, g, src, D, m, d_out, nka, io.ktile(2));
  __syncthreads();
  load_frags(f0, smem, 0, 0, ad);
#define ECHOKV_KT(STAGE, ST) \
  k_tile<SWAP, PACKED, STAGE, true, true>(acc, f0, f1, ST, smem, ad, g, src, D, m, d_out, nka, io.ktile(kt + 3))
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    ECHOKV_KT(0, sb);
    ++kt;
    ECHOKV_KT(1, sa);
    --kt;
  }
  if (kt < nk) ECHOKV_KT(0, sb);
#undef ECHOKV_KT
}

// Workgroup id -> (token tile, column tile).  Consecutive workgroup ids go to
// different XCDs, so each XCD is given one contiguous range of logical tiles:
// the column tiles of a token tile then hit the same L2 copy of X.
__device__ __forceinline__ bool tile_of_block(const Args& a, int& ttile, int& ctile) {
  const int per_xcd = (a.n_tiles + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= a.n_tiles) return false;
  ttile = logical / a.n_col_tiles;
  ctile = logical % a.n_col_tiles;
  return true;
}

// Queries of the tile's heads -> LDS as fp32, pre-scaled by the softmax scale.
template <int HD, typename T>
__device__ __forceinline__ void load_queries(EpiSmem& e, const T* q, int b, int H_q, int G,
                                             int kvh0, float scale, int tid) {
  const int H_kv = H_q / G;
  for (int idx = tid; idx < (BN / HD) * G * HD; idx += NTHREADS) {
    const int c = idx % HD, pg = idx / HD;       // pg = head_in_tile * G + g
    const int kvh = kvh0 + pg / G;
    float v = 0.f;
    if (kvh < H_kv) v = Elem<T>::to_f32(q[((int64_t)b * H_q + kvh * G + pg % G) * HD + c]) * scale;
    e.q[pg * HD + c] = v;
  }
}

// After the K pass: acc[ci][ji] holds K_hat^T (rows = head dims of the wave's
// 128 columns, lanes = tokens).  Scores (Eq. 7), masked beyond L, then the
// wave's softmax numerators -> e.p, (max, sum) -> e.ml, per (head, query head).
// Keeps the accumulators in the accumulation registers for the duration of an
// epilogue loop body: without it the compiler copies all 256 of them to
// ordinary registers ahead of the loop over query heads and spills whatever
// else is live (e.g. a prefetched k-tile).
__device__ __forceinline__ void pin_acc(floatx16_t (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+a"(acc[i][j]));
}

// Extras of the score epilogue: rotary tables (null: none) and the token range [lo, hi) of the
// sequence that counts (tokens outside are masked: past the end, or held by the window).
struct KExtra {
  const float* cos; const float* sin;
  int lo, hi;
};
__device__ __forceinline__ KExtra make_kextra(const float* cos, const float* sin, int n_sink,
                                              int n_recent, int L) {
  KExtra x;
  x.cos = cos; x.sin = sin;
  const bool win = n_sink + n_recent > 0;
  x.lo = win ? min(n_sink, L) : 0;
  x.hi = win ? max(x.lo, L - n_recent) : L;
  return x;
}

// Softmax numerators of one (head, query head) pair from the lane-partial scores s[4]
// (token ji * 32 + lane % 32; the two lane halves hold the two halves of the head dims).
__device__ __forceinline__ void score_tail(float (&s)[4], EpiSmem& e, int wave, int lane, int pair,
                                           int jw0, const KExtra& x) {
  const int lr = lane & 31, lh = lane >> 5;
  float mx = -INFINITY;
#pragma unroll
  for (int ji = 0; ji < 4; ++ji) {
    s[ji] += __shfl_xor(s[ji], 32, 64);
    const int tok = jw0 + ji * 32 + lr;
    if (tok < x.lo || tok >= x.hi) s[ji] = -INFINITY;
    mx = fmaxf(mx, s[ji]);
  }
  mx = wave_max(mx, 32);
  float sum = 0.f;
  float* pp = e.p[wave][pair];
#pragma unroll
  for (int ji = 0; ji < 4; ++ji) {
    const float p = (s[ji] == -INFINITY) ? 0.f : __expf(s[ji] - mx);
    sum += p;
    if (lh == 0) pp[ji * 32 + lr] = p;
  }
  sum = wave_sum(sum, 32);
  if (lane == 0) { e.ml[wave][pair][0] = mx; e.ml[wave][pair][1] = sum; }
}

// `tail(s, hw, g)` receives the lane-partial scores s[4] of head hw of the wave's tile and
// query head g of its group (token ji * 32 + lane % 32; add the other lane half for the total).
template <int HD, bool ROPE, class Tail>
__device__ __forceinline__ void k_scores(floatx16_t (&acc)[4][4], EpiSmem& e, int G,
                                         int wave, int lane, int jw0, int L, const KExtra& x,
                                         Tail tail) {
  constexpr int HPW = WN / HD, CBH = HD / 32;
  const int wc = wave & 1, lr = lane & 31, lh = lane >> 5;
  if constexpr (!ROPE) {
#pragma unroll
    for (int hw = 0; hw < HPW; ++hw) {
      for (int g = 0; g < G; ++g) {
        pin_acc(acc);
        const float* qs = &e.q[((wc * HPW + hw) * G + g) * HD];
        float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cb = 0; cb < CBH; ++cb) {
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const float4 qv = *reinterpret_cast<const float4*>(qs + cb * 32 + r4 * 8 + lh * 4);
#pragma unroll
            for (int ji = 0; ji < 4; ++ji) {
              const floatx16_t& c = acc[hw * CBH + cb][ji];
              s[ji] = fmaf(qv.x, c[r4 * 4 + 0], s[ji]);
              s[ji] = fmaf(qv.y, c[r4 * 4 + 1], s[ji]);
              s[ji] = fmaf(qv.z, c[r4 * 4 + 2], s[ji]);
              s[ji] = fmaf(qv.w, c[r4 * 4 + 3], s[ji]);
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        tail(s, hw, g);
      }
    }
  } else {
    // Rotary embedding of the rebuilt key at its token's position, folded into the dot
    // product: feature c pairs with c + HD/2, which this lane holds HD/64 column blocks
    // further on.  With a = k_c, b = k_{c+HD/2}:
    //   q_c (a cos - b sin) + q_{c+HD/2} (b cos + a sin)
    //     = cos (a q_c + b q_{c+HD/2}) + sin (a q_{c+HD/2} - b q_c)
    // The accumulators are only read.  Masked tokens borrow the last valid table row.  The
    // table values and the accumulator reads of a (token block, column block) are shared by
    // the query heads of the group: the loop over them is innermost, unrolled to the
    // largest group size with a uniform skip.
    constexpr int HB = CBH / 2;
#pragma unroll
    for (int hw = 0; hw < HPW; ++hw) {
      float s[MAXPAIR][4];
#pragma unroll
      for (int g = 0; g < MAXPAIR; ++g)
#pragma unroll
        for (int ji = 0; ji < 4; ++ji) s[g][ji] = 0.f;
#pragma unroll
      for (int ji = 0; ji < 4; ++ji) {
        const int pos = min(jw0 + ji * 32 + lr, L - 1);
        const float* cr = x.cos + (int64_t)pos * (HD / 2) + lh * 4;
        const float* sr = x.sin + (int64_t)pos * (HD / 2) + lh * 4;
#pragma unroll
        for (int cb = 0; cb < HB; ++cb) {
          pin_acc(acc);
          float cc[16], ss[16], ka[16], kb[16];
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const float4 c4 = *reinterpret_cast<const float4*>(cr + cb * 32 + r4 * 8);
            const float4 s4 = *reinterpret_cast<const float4*>(sr + cb * 32 + r4 * 8);
            cc[r4 * 4] = c4.x; cc[r4 * 4 + 1] = c4.y; cc[r4 * 4 + 2] = c4.z; cc[r4 * 4 + 3] = c4.w;
            ss[r4 * 4] = s4.x; ss[r4 * 4 + 1] = s4.y; ss[r4 * 4 + 2] = s4.z; ss[r4 * 4 + 3] = s4.w;
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            ka[r] = acc[hw * CBH + cb][ji][r];
            kb[r] = acc[hw * CBH + cb + HB][ji][r];
          }
#pragma unroll
          for (int g = 0; g < MAXPAIR; ++g) {
            if (g < G) {
              const float* qs = &e.q[((wc * HPW + hw) * G + g) * HD];
#pragma unroll
              for (int r4 = 0; r4 < 4; ++r4) {
                const float4 qa = *reinterpret_cast<const float4*>(qs + cb * 32 + r4 * 8 + lh * 4);
                const float4 qb = *reinterpret_cast<const float4*>(qs + (cb + HB) * 32 + r4 * 8 + lh * 4);
                const float q0[4] = {qa.x, qa.y, qa.z, qa.w}, q1[4] = {qb.x, qb.y, qb.z, qb.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                  const float a = ka[r4 * 4 + i], b = kb[r4 * 4 + i];
                  const float t1 = fmaf(a, q0[i], b * q1[i]);
                  const float t2 = fmaf(a, q1[i], -b * q0[i]);
                  s[g][ji] = fmaf(cc[r4 * 4 + i], t1, fmaf(ss[r4 * 4 + i], t2, s[g][ji]));
                }
              }
            }
          }
          asm volatile("" ::: "memory");       // keep the table loads of later rounds from piling up
          __builtin_amdgcn_sched_barrier(0);
        }
      }
#pragma unroll
      for (int g = 0; g < MAXPAIR; ++g)
        if (g < G) tail(s[g], hw, g);
    }
  }
}

// Scores -> this wave's softmax numerators in LDS (the fused kernel's score epilogue).
template <int HD, bool ROPE>
__device__ __forceinline__ void k_epilogue(floatx16_t (&acc)[4][4], EpiSmem& e, int G,
                                           int wave, int lane, int jw0, int L, const KExtra& x) {
  k_scores<HD, ROPE>(acc, e, G, wave, lane, jw0, L, x,
                     [&](float (&s)[4], int hw, int g) { score_tail(s, e, wave, lane, hw * G + g, jw0, x); });
}

// After the V pass: acc[ji][ci] holds V_hat (rows = tokens, lanes = head dims).
// sum_j p_j v_hat_j per (head, query head) -> one split-K partial per wave.
template <int HD>
__device__ __forceinline__ void v_epilogue(floatx16_t (&acc)[4][4], const EpiSmem& e, int G,
                                           int wave, int lane, int slot, int H_q, int kvh_wave0,
                                           float* part_o, float* part_ml) {
  constexpr int HPW = WN / HD, CBH = HD / 32;
  const int lr = lane & 31, lh = lane >> 5;
  const int H_kv = H_q / G;
#pragma unroll
  for (int hw = 0; hw < HPW; ++hw) {
    const int kvh = kvh_wave0 + hw;
    if (kvh >= H_kv) continue;
    for (int g = 0; g < G; ++g) {
      pin_acc(acc);
      const float* pp = e.p[wave][hw * G + g];
      float o[CBH];
#pragma unroll
      for (int cb = 0; cb < CBH; ++cb) o[cb] = 0.f;
#pragma unroll
      for (int ji = 0; ji < 4; ++ji) {
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 pv = *reinterpret_cast<const float4*>(pp + ji * 32 + r4 * 8 + lh * 4);
#pragma unroll
          for (int cb = 0; cb < CBH; ++cb) {
            const floatx16_t& c = acc[ji][hw * CBH + cb];
            o[cb] = fmaf(pv.x, c[r4 * 4 + 0], o[cb]);
            o[cb] = fmaf(pv.y, c[r4 * 4 + 1], o[cb]);
            o[cb] = fmaf(pv.z, c[r4 * 4 + 2], o[cb]);
            o[cb] = fmaf(pv.w, c[r4 * 4 + 3], o[cb]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      const int64_t ph = (int64_t)slot * H_q + kvh * G + g;
#pragma unroll
      for (int cb = 0; cb < CBH; ++cb) {
        o[cb] += __shfl_xor(o[cb], 32, 64);
        if (lh == 0) part_o[ph * HD + cb * 32 + lr] = o[cb];
      }
      if (lane == 0) {
        part_ml[ph * 2] = e.ml[wave][hw * G + g][0];
        part_ml[ph * 2 + 1] = e.ml[wave][hw * G + g][1];
      }
    }
  }
}

template <int HD, bool PACKED, bool ROPE>
__global__ __launch_bounds__(NTHREADS) void fused_decode_kernel(Args a, SeqMeta meta) {
  __shared__ Smem sm;
  char* smem = reinterpret_cast<char*>(&sm);
  int ttile, ctile;
  if (!tile_of_block(a, ttile, ctile)) return;
  const int b = find_seq(meta.tbase, meta.n, ttile);
  const int L = meta.len[b];
  const int j0 = (ttile - meta.tbase[b]) * BM;
  const int n0 = ctile * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1;

  // rows past the end of the sequence are clamped onto its last valid token,
  // so that masked tokens still contribute finite numbers
  const int last = min(BM, L - j0) - 1;
  const int64_t row0 = meta.start[b] + j0;
  const int nclamp = a.d_out - n0 - 8;     // last readable 8-column block of this tile
  load_queries<HD>(sm.e, a.q, b, a.H_q, a.G, a.n_ret_heads + n0 / HD, a.scale, tid);

  floatx16_t acc[4][4];
  const int rot = (ttile * 3) % ((a.D + a.m) / BK);
  // W tile base: column n0 of row-major W, or row n0 of the packed transpose
  const int64_t woff = PACKED ? (int64_t)n0 * (a.D + a.m) : n0;
  Stage sa, sb;
  PassIo io;
  // ---- K_hat^T = W_K^T X^T (gemm_pass begins with a barrier, which publishes e.q)
  make_io(io, a, a.xa[0] + row0 * a.D, a.xr[0] + row0 * a.m, a.w[0] + woff, last, nclamp, tid, rot);
  pass_prefetch<PACKED>(sa, io, a);
  gemm_pass<true, PACKED>(acc, smem, a, io, sa, sb, tid);
  // the V pass's first tiles are requested now and land while the scores are worked out
  make_io(io, a, a.xa[1] + row0 * a.D, a.xr[1] + row0 * a.m, a.w[1] + woff, last, nclamp, tid, rot);
  pass_prefetch<PACKED>(sa, io, a);
  const int jw0 = j0 + wt * WM;                 // first token of this wave
  k_epilogue<HD, ROPE>(acc, sm.e, a.G, wave, lane, jw0, L,
                       make_kextra(a.rope_cos, a.rope_sin, a.n_sink, a.n_recent, L));
  // ---- V_hat = X W_V (e.p / e.ml are wave-private; the pass's barriers order them anyway)
  gemm_pass<false, PACKED>(acc, smem, a, io, sa, sb, tid);
  if (jw0 >= L) return;                          // wave has no valid token: no partial
  v_epilogue<HD>(acc, sm.e, a.G, wave, lane, meta.sbase[b] + jw0 / kSlotTokens, a.H_q,
                 a.n_ret_heads + (n0 + wc * WN) / HD, a.part_o, a.part_ml);
}

// Key half of the fused kernel on its own: K_hat^T of the tile, then the scaled scores of
// every (head, query head) of the tile written to S^T (base-2 logits: the caller folds log2 e
// into the scale).  Used when the value side is evaluated in the other association order
// (sum_j p_j x^V_j first, W_V afterwards), which stays valid under a rotary embedding.
template <int HD, bool ROPE>
__global__ __launch_bounds__(NTHREADS) void fused_kscores_kernel(Args a, SeqMeta meta) {
  __shared__ Smem sm;
  char* smem = reinterpret_cast<char*>(&sm);
  int ttile, ctile;
  if (!tile_of_block(a, ttile, ctile)) return;
  const int b = find_seq(meta.tbase, meta.n, ttile);
  const int L = meta.len[b];
  const int j0 = (ttile - meta.tbase[b]) * BM;
  const int n0 = ctile * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1, lr = lane & 31, lh = lane >> 5;
  const int last = min(BM, L - j0) - 1;
  const int64_t row0 = meta.start[b] + j0;
  const int nclamp = a.d_out - n0 - 8;
  load_queries<HD>(sm.e, a.q, b, a.H_q, a.G, a.n_ret_heads + n0 / HD, a.scale, tid);
  floatx16_t acc[4][4];
  Stage sa, sb;
  PassIo io;
  make_io(io, a, a.xa[0] + row0 * a.D, a.xr[0] + row0 * a.m, a.w[0] + n0, last, nclamp, tid,
          (ttile * 3) % ((a.D + a.m) / BK));
  pass_prefetch<false>(sa, io, a);
  gemm_pass<true, false>(acc, smem, a, io, sa, sb, tid);
  const int jw0 = j0 + wt * WM;
  if (jw0 >= L) return;
  constexpr int HPW = WN / HD;
  const int kvh0 = a.n_ret_heads + (n0 + wc * WN) / HD;       // first KV head of this wave's columns
  const int H_kv = a.H_q / a.G;
  float* srow = a.s_out + (int64_t)meta.sbase[b] * kSlotTokens + jw0 + lr;
  KExtra x = make_kextra(a.rope_cos, a.rope_sin, 0, 0, L);
  if (HPW == 1 && kvh0 >= H_kv) return;      // columns past the last head (an exit, not a branch to rejoin)
  k_scores<HD, ROPE>(acc, sm.e, a.G, wave, lane, jw0, L, x, [&](float (&s)[4], int hw, int g) {
    if (HPW > 1 && kvh0 + hw >= H_kv) return;
    float* dst = srow + (int64_t)((kvh0 + hw) * a.G + g) * a.s_ld;
#pragma unroll
    for (int ji = 0; ji < 4; ++ji) {
      const float v = s[ji] + __shfl_xor(s[ji], 32, 64);
      if (lh == 0 && jw0 + ji * 32 + lr < L) dst[ji * 32] = v;
    }
  });
}

// Stand-alone predictor product (Eq. 3) with the same main loop: K_hat or V_hat
// (blockIdx.y) of the tile is rounded to bf16 and stored at
// out[row, col0 + column].  Output row = sbase[b]*kSlotTokens + j.  With an
// activation it is the first layer of the one-hidden-layer predictor
// (Appendix "Prediction Network Architecture").
template <int ACT, bool OUT32 = false>   // activation before rounding: 0 none, 1 ReLU, 2 SiLU; OUT32: fp32 output
__global__ __launch_bounds__(NTHREADS) void recon_mfma_kernel(Args a, SeqMeta meta) {
  __shared__ Smem sm;
  char* smem = reinterpret_cast<char*>(&sm);
  int ttile, ctile;
  if (!tile_of_block(a, ttile, ctile)) return;
  const int which = blockIdx.y;
  const int b = find_seq(meta.tbase, meta.n, ttile);
  const int L = meta.len[b];
  const int j0 = (ttile - meta.tbase[b]) * BM;
  const int n0 = ctile * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wt = wave >> 1, wc = wave & 1;
  const int lr = lane & 31, lh = lane >> 5;
  const int last = min(BM, L - j0) - 1;
  const int64_t row0 = meta.start[b] + j0;
  const int nclamp = a.d_out - n0 - 8;
  floatx16_t acc[4][4];
  Stage sa, sb;
  PassIo io;
  make_io(io, a, a.xa[which] + row0 * a.D, a.xr[which] + row0 * a.m, a.w[which] + n0, last, nclamp,
          tid, (ttile * 3) % ((a.D + a.m) / BK));
  pass_prefetch<false>(sa, io, a);
  gemm_pass<false, false>(acc, smem, a, io, sa, sb, tid);
  // activation of a hidden layer (a compile-time choice: a run-time branch over 256 live
  // accumulators costs hundreds of spilled registers)
  if constexpr (ACT == 1) {
#pragma unroll
    for (int ji = 0; ji < 4; ++ji)
#pragma unroll
      for (int ci = 0; ci < 4; ++ci)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ji][ci][r] = fmaxf(acc[ji][ci][r], 0.f);
  } else if constexpr (ACT == 2) {
#pragma unroll
    for (int ji = 0; ji < 4; ++ji)
#pragma unroll
      for (int ci = 0; ci < 4; ++ci)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[ji][ci][r] = acc[ji][ci][r] / (1.f + __expf(-acc[ji][ci][r]));
  }
  bf16_t* out = a.out[which];
  const int64_t orow0 = (int64_t)meta.sbase[b] * kSlotTokens;
#pragma unroll
  for (int ji = 0; ji < 4; ++ji) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = j0 + wt * WM + ji * 32 + (r >> 2) * 8 + lh * 4 + (r & 3);
      if (j >= L) continue;
#pragma unroll
      for (int ci = 0; ci < 4; ++ci) {
        const int c = n0 + wc * WN + ci * 32 + lr;
        if (c < a.d_out) {
          if constexpr (OUT32) reinterpret_cast<float*>(out)[(orow0 + j) * a.ldo + a.col0 + c] = acc[ji][ci][r];
          else out[(orow0 + j) * a.ldo + a.col0 + c] = f32_to_bf16(acc[ji][ci][r]);
        }
      }
    }
  }
}

}  // namespace fused

// ---- host-side launchers ------------------------------------------------------------
// Paper-faithful extras of a decode call as the launchers take them (all zero: off).
struct KvExtras {
  const float* rope_cos = nullptr; const float* rope_sin = nullptr;
  int n_sink = 0, n_recent = 0;
};

template <typename T> inline bool fused_decode_supported(int d, int G) {
  return (d == 64 || d == 128) && (128 / d) * G <= fused::MAXPAIR;
}
template <typename T> inline bool recon_mfma_supported() { return sizeof(T) == 2; }

inline int fused_fill_tiles(SeqMeta& mt) {
  int acc = 0;
  for (int b = 0; b < mt.n; ++b) { mt.tbase[b] = acc; acc += (mt.len[b] + fused::BM - 1) / fused::BM; }
  mt.tbase[mt.n] = acc;
  return acc;
}

template <typename T>
inline int launch_fused_decode(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                               float scale, const T* ka,
                               const T* va, const T* kr, const T* vr, const T* wk, const T* wv,
                               const T* q, float* part_o, float* part_ml, SeqMeta& mt,
                               int* fused_step, hipStream_t st, bool packed = false,
                               const KvExtras& ex = KvExtras(), int x_width = 0) {
  if constexpr (sizeof(T) != 2) {
    return 6;
  } else {
    fused::Args a;
    a.rope_cos = ex.rope_cos; a.rope_sin = ex.rope_sin; a.n_sink = ex.n_sink; a.n_recent = ex.n_recent;
    a.s_out = nullptr; a.s_ld = 0;
    a.xa[0] = ka; a.xa[1] = va; a.xr[0] = kr; a.xr[1] = vr; a.w[0] = wk; a.w[1] = wv;
    a.q = q; a.part_o = part_o; a.part_ml = part_ml;
    a.out[0] = a.out[1] = nullptr; a.ldo = 0; a.col0 = 0;
    a.D = H_kv * d; a.m = m; a.d_out = d_out; a.H_q = H_q; a.G = H_q / H_kv;
    if (x_width > 0) { a.D = x_width; a.m = 0; }     // predictor input = one matrix of that width (ka / va)
    a.n_ret_heads = n_ret_heads; a.scale = scale;
    a.n_col_tiles = (a.d_out + fused::BN - 1) / fused::BN;
    a.n_tiles = fused_fill_tiles(mt) * a.n_col_tiles;
    const int grid = ((a.n_tiles + 7) / 8) * 8;
    const dim3 g(grid), blk(fused::NTHREADS);
    const bool rope = ex.rope_cos != nullptr;
#define ECHOKV_FUSED_CASE(HD_, PK_) \
    do { if (rope) hipLaunchKernelGGL((fused::fused_decode_kernel<HD_, PK_, true>), g, blk, 0, st, a, mt); \
         else hipLaunchKernelGGL((fused::fused_decode_kernel<HD_, PK_, false>), g, blk, 0, st, a, mt); } while (0)
    if (d == 128 && packed) ECHOKV_FUSED_CASE(128, true);
    else if (d == 128) ECHOKV_FUSED_CASE(128, false);
    else if (packed) ECHOKV_FUSED_CASE(64, true);
    else ECHOKV_FUSED_CASE(64, false);
#undef ECHOKV_FUSED_CASE
    if (hipGetLastError() != hipSuccess) return 7;
    *fused_step = 1;
    return 0;
  }
}

// Scores of the predicted heads -> s_out (see fused_kscores_kernel).  `scale` must already
// include log2(e).
template <typename T>
inline int launch_fused_kscores(int H_q, int H_kv, int d, int m, int d_out, int n_ret_heads,
                                float scale, const T* ka, const T* kr, const T* wk, const T* q,
                                float* s_out, int64_t s_ld, SeqMeta& mt, hipStream_t st,
                                const KvExtras& ex = KvExtras()) {
  if constexpr (sizeof(T) != 2) {
    return 6;
  } else {
    fused::Args a;
    a.xa[0] = a.xa[1] = ka; a.xr[0] = a.xr[1] = kr; a.w[0] = a.w[1] = wk;
    a.q = q; a.part_o = nullptr; a.part_ml = nullptr;
    a.out[0] = a.out[1] = nullptr; a.ldo = 0; a.col0 = 0;
    a.D = H_kv * d; a.m = m; a.d_out = d_out; a.H_q = H_q; a.G = H_q / H_kv;
    a.n_ret_heads = n_ret_heads; a.scale = scale;
    a.rope_cos = ex.rope_cos; a.rope_sin = ex.rope_sin; a.n_sink = 0; a.n_recent = 0;
    a.s_out = s_out; a.s_ld = s_ld;
    a.n_col_tiles = (a.d_out + fused::BN - 1) / fused::BN;
    a.n_tiles = fused_fill_tiles(mt) * a.n_col_tiles;
    const dim3 g(((a.n_tiles + 7) / 8) * 8), blk(fused::NTHREADS);
    const bool rope = ex.rope_cos != nullptr;
    if (d == 128 && rope) hipLaunchKernelGGL((fused::fused_kscores_kernel<128, true>), g, blk, 0, st, a, mt);
    else if (d == 128) hipLaunchKernelGGL((fused::fused_kscores_kernel<128, false>), g, blk, 0, st, a, mt);
    else if (rope) hipLaunchKernelGGL((fused::fused_kscores_kernel<64, true>), g, blk, 0, st, a, mt);
    else hipLaunchKernelGGL((fused::fused_kscores_kernel<64, false>), g, blk, 0, st, a, mt);
    if (hipGetLastError() != hipSuccess) return 7;
    return 0;
  }
}

// K_hat and V_hat of the sequences in `mt` -> out_k / out_v [rows, ldo] at
// column col0, output row = sbase[b]*kSlotTokens + j.  d_out = width of W.
template <typename T>
inline int launch_recon_mfma(int D, int m, int d_out, const T* ka, const T* va, const T* kr, const T* vr,
                             const T* wk, const T* wv, T* out_k, T* out_v, int64_t ldo, int col0,
                             SeqMeta& mt, hipStream_t st, int act = 0, bool out_f32 = false) {
  if constexpr (sizeof(T) != 2) {
    return 6;
  } else {
    fused::Args a;
    a.xa[0] = ka; a.xa[1] = va; a.xr[0] = kr; a.xr[1] = vr; a.w[0] = wk; a.w[1] = wv;
    a.q = nullptr; a.part_o = nullptr; a.part_ml = nullptr;
    a.rope_cos = a.rope_sin = nullptr; a.n_sink = a.n_recent = 0; a.s_out = nullptr; a.s_ld = 0;
    a.out[0] = out_k; a.out[1] = out_v; a.ldo = ldo; a.col0 = col0;
    a.D = D; a.m = m; a.d_out = d_out; a.H_q = 0; a.G = 1; a.n_ret_heads = 0; a.scale = 0.f;
    a.n_col_tiles = (a.d_out + fused::BN - 1) / fused::BN;
    a.n_tiles = fused_fill_tiles(mt) * a.n_col_tiles;
    const int grid = ((a.n_tiles + 7) / 8) * 8;
    const dim3 g(grid, 2), blk(fused::NTHREADS);
    if (out_f32) hipLaunchKernelGGL((fused::recon_mfma_kernel<0, true>), g, blk, 0, st, a, mt);
    else if (act == 1) hipLaunchKernelGGL(fused::recon_mfma_kernel<1>, g, blk, 0, st, a, mt);
    else if (act == 2) hipLaunchKernelGGL(fused::recon_mfma_kernel<2>, g, blk, 0, st, a, mt);
    else hipLaunchKernelGGL(fused::recon_mfma_kernel<0>, g, blk, 0, st, a, mt);
    if (hipGetLastError() != hipSuccess) return 7;
    return 0;
  }
}

}  // namespace echokv
