// Bandwidth-bound kernels of the EchoKV path: cache append (strided row copy),
// split-K streaming decode attention over stored heads, and the split merge.
// Also a plain FMA-tiled predictor GEMM used by the unfused comparison path
// and by the fp32 configuration.
#pragma once
#include "common.h"

namespace echokv {

// ---------------------------------------------------------------------------
// Row copy: dst[drow0(r) , 0:width) = src[r, 0:width) in 16-byte pieces.
// Cache append keeps only the first `width` flattened dims of each new row
// (Eq. 1 for an anchor layer, Eq. 2 for a target layer).
// meta.tbase = prefix sum of new rows per sequence; destination row of new row
// r of sequence b is start[b] + len[b] + (r - tbase[b]) (len = length BEFORE).
// blockIdx.y selects K (0) or V (1).
// ---------------------------------------------------------------------------
struct CopyArgs {
  const char* src[2];
  char* dst[2];
  int64_t src_row_bytes;
  int64_t dst_row_bytes;   // == bytes copied per row
  int32_t rows;
};

__global__ __launch_bounds__(256) void append_rows_kernel(CopyArgs a, SeqMeta meta) {
  const int which = blockIdx.y;
  const int pieces = (int)(a.dst_row_bytes >> 4);
  for (int r = blockIdx.x; r < a.rows; r += gridDim.x) {
    const int b = find_seq(meta.tbase, meta.n, r);
    const int64_t drow = meta.start[b] + meta.len[b] + (r - meta.tbase[b]);
    const uint4* s = reinterpret_cast<const uint4*>(a.src[which] + (int64_t)r * a.src_row_bytes);
    uint4* d = reinterpret_cast<uint4*>(a.dst[which] + drow * a.dst_row_bytes);
    for (int i = threadIdx.x; i < pieces; i += blockDim.x) d[i] = s[i];
  }
}

// ---------------------------------------------------------------------------
// Uncompressed window of the target layer (the first n_sink positions and a
// ring of the n_recent latest, Sec. "Experimental Setting", paragraph "Implement details"): position p lives in
// row p (p < n_sink) or n_sink + (p - n_sink) % n_recent.
// ---------------------------------------------------------------------------
struct Window {
  int32_t n_sink, n_recent;      // n_sink + n_recent == 0: no window
  __host__ __device__ int rows() const { return n_sink + n_recent; }
  __host__ __device__ bool on() const { return n_sink + n_recent > 0; }
  // compressed-cache tokens [lo, hi) of a length-L sequence are NOT in the window
  __host__ __device__ int lo(int L) const { return on() ? (n_sink < L ? n_sink : L) : 0; }
  __host__ __device__ int hi(int L) const {
    if (!on()) return L;
    const int h = L - n_recent, l = lo(L);
    return h > l ? h : l;
  }
  __host__ __device__ int row_of(int p) const { return p < n_sink ? p : n_sink + (p - n_sink) % n_recent; }
  // position held by window row w of a length-L sequence, or -1 if the row is empty / stale
  __host__ __device__ int pos_of(int w, int L) const {
    if (w < n_sink) return w < L ? w : -1;
    if (n_recent == 0) return -1;
    const int t = L - 1 - n_sink, r = w - n_sink;      // ring coordinates of the last token, of the row
    if (t < 0) return -1;
    int back = (t - r) % n_recent;
    if (back < 0) back += n_recent;
    return t - back >= 0 ? n_sink + t - back : -1;
  }
};

// New full-width rows -> window.  meta: start[b] = length BEFORE the append, len[b] = new rows,
// tbase = prefix sum of new rows.  A new row is written only if it is still inside the window
// once all of the call's rows are in, so every window row has one writer.  blockIdx.y: K / V.
struct WinAppendArgs {
  const char* src[2];
  char* dst[2];
  int64_t row_bytes;
  int32_t rows, seq0;
  Window win;
};
__global__ __launch_bounds__(256) void window_append_kernel(WinAppendArgs a, SeqMeta meta) {
  const int which = blockIdx.y;
  const int pieces = (int)(a.row_bytes >> 4);
  for (int r = blockIdx.x; r < a.rows; r += gridDim.x) {
    const int b = find_seq(meta.tbase, meta.n, r);
    const int p = (int)meta.start[b] + (r - meta.tbase[b]);
    const int L_after = (int)meta.start[b] + meta.len[b];
    if (p >= a.win.n_sink && p < L_after - a.win.n_recent) continue;
    const int64_t drow = (int64_t)(a.seq0 + b) * a.win.rows() + a.win.row_of(p);
    const uint4* s = reinterpret_cast<const uint4*>(a.src[which] + (int64_t)r * a.row_bytes);
    uint4* d = reinterpret_cast<uint4*>(a.dst[which] + drow * a.row_bytes);
    for (int i = threadIdx.x; i < pieces; i += blockDim.x) d[i] = s[i];
  }
}

// Plain streaming read of a buffer, 8 independent 16-byte loads in flight per thread: the
// yardstick the HBM-bound kernels are compared with (measurement aid, not part of the method).
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* p, int64_t n16_per_block,
                                                          uint32_t* sink) {
  const uint4* base = p + (int64_t)blockIdx.x * n16_per_block + threadIdx.x;
  uint4 acc = make_uint4(0u, 0u, 0u, 0u);
  for (int64_t o = 0; o < n16_per_block; o += 8 * 256) {
    uint4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = base[o + j * 256];
#pragma unroll
    for (int j = 0; j < 8; ++j) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u && sink) *sink = 1u;   // keeps the loads alive
}

// Plain 2-D copy of `rows` rows (used to place the retained dims in front of
// the predicted ones, Eq. 6).  blockIdx.y selects K or V.
struct Copy2dArgs {
  const char* src[2];
  char* dst[2];
  int64_t src_row_bytes, dst_row_bytes, copy_bytes;
  int64_t rows;
};
__global__ __launch_bounds__(256) void copy2d_kernel(Copy2dArgs a) {
  const int which = blockIdx.y;
  const int pieces = (int)(a.copy_bytes >> 4);
  for (int64_t r = blockIdx.x; r < a.rows; r += gridDim.x) {
    const uint4* s = reinterpret_cast<const uint4*>(a.src[which] + r * a.src_row_bytes);
    uint4* d = reinterpret_cast<uint4*>(a.dst[which] + r * a.dst_row_bytes);
    for (int i = threadIdx.x; i < pieces; i += blockDim.x) d[i] = s[i];
  }
}

// In-place narrowing of rows [r0, r1) of a row-major matrix from src_row_bytes to the first
// dst_row_bytes of each row, both at `base` (the full -> compressed switch of a target layer done
// where the full cache lies).  Every destination byte sits at or below the source byte it comes
// from, so walking the 16-byte pieces in (row, piece) order never overwrites a piece that is still
// to be read -- as long as the pieces of one round have all been read before any of them is
// written.  One workgroup per matrix (blockIdx.x = K or V) takes rounds of 256 x 16 pieces: load
// all into registers, wait for the data, barrier, store.  Used for the first rows only; further on
// source and destination of whole row ranges no longer overlap and plain copies take over.
struct CompactArgs {
  char* base[2];
  int64_t src_row_bytes, dst_row_bytes;
  int64_t r0, r1;
};
__global__ __launch_bounds__(256) void compact_rows_seq_kernel(CompactArgs a) {
  char* base = a.base[blockIdx.x];
  const int64_t ppr = a.dst_row_bytes >> 4;               // pieces per row
  const int64_t p_end = a.r1 * ppr;
  for (int64_t p0 = a.r0 * ppr; p0 < p_end; p0 += 256 * 16) {
    uint4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int64_t p = p0 + j * 256 + threadIdx.x;
      if (p < p_end) {
        const int64_t row = p / ppr, c = p - row * ppr;
        v[j] = *reinterpret_cast<const uint4*>(base + row * a.src_row_bytes + c * 16);
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0070);      // vmcnt(0): this round's pieces are in registers
    __syncthreads();                          // ... for every wave, before any of them is overwritten
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int64_t p = p0 + j * 256 + threadIdx.x;
      if (p < p_end) {
        const int64_t row = p / ppr, c = p - row * ppr;
        *reinterpret_cast<uint4*>(base + row * a.dst_row_bytes + c * 16) = v[j];
      }
    }
  }
}

// ---------------------------------------------------------------------------
// dst[c, r] = src[r, c] for a row-major [R, C] matrix (row pitch ld_src): 64x64 tiles through LDS.
// Used once per weight matrix to lay W out as [d_out, d_in] (k-contiguous rows),
// the layout an MFMA operand wants.  grid = (ceil(C/64), ceil(R/64)).
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T* src, T* dst, int R, int C,
                                                        int64_t ld_src) {
  __shared__ T tile[64][65];
  const int c0 = blockIdx.x * 64, r0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4)
    if (r0 + i < R && c0 + tx < C) tile[i][tx] = src[(int64_t)(r0 + i) * ld_src + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 64; i += 4)
    if (c0 + i < C && r0 + tx < R) dst[(int64_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

// ---------------------------------------------------------------------------
// Extended weights for a target layer whose retained prefix ends inside a head
// (m = g0*d + r, r > 0): out[k, v] = (k == sel0 + v) for v < r, W[k, v - r] else,
// out being [d_in, d_out + r] row-major.  The r selector columns make the
// predictor product reproduce the split head's retained dims bit for bit, so
// the attention kernels can treat that head as fully predicted (Eq. 6 concat).
// grid = (d_in, 2): one block per input row, blockIdx.y = K or V.
// ---------------------------------------------------------------------------
template <typename T>
struct AugArgs {
  const T* w[2];
  T* out[2];
  int32_t d_in, d_out, r, sel0;
};
template <typename T>
__global__ __launch_bounds__(256) void augment_weights_kernel(AugArgs<T> a) {
  const int k = blockIdx.x, which = blockIdx.y;
  const T* src = a.w[which] + (int64_t)k * a.d_out;
  T* dst = a.out[which] + (int64_t)k * (a.d_out + a.r);
  for (int v = threadIdx.x; v < a.d_out + a.r; v += blockDim.x)
    dst[v] = (v < a.r) ? Elem<T>::from_f32(k == a.sel0 + v ? 1.0f : 0.0f) : src[v - a.r];
}

// ---------------------------------------------------------------------------
// Predictor product with ordinary FMAs (Eq. 3): for the tokens of each
// sequence, out[row, col0 + c] = sum_k X[j,k] W[k,c], X = [anchor row ; retained row].
// 64x64 output tile, 256 threads, 4x4 outputs each, fp32 accumulation.
// blockIdx.z selects K (0) or V (1).  Output rows: out_row0[b] + j with
// out_row0 = sbase[b]*kSlotTokens (workspace) or an explicit single offset.
// ---------------------------------------------------------------------------
template <typename T>
struct GemmArgs {
  const T* xa[2];   // anchor cache  [pool, D]
  const T* xr[2];   // retained cache [pool, m]
  const T* w[2];    // [d_in, d_out]
  T* out[2];
  int32_t D, m, d_out;
  int64_t ldo;      // output row stride (elements)
  int32_t col0;     // first output column (elements)
  int32_t rows_from_slots;  // 1: output row = sbase[b]*kSlotTokens + j ; 0: row = j
};

template <typename T>
__global__ __launch_bounds__(256) void recon_fma_kernel(GemmArgs<T> a, SeqMeta meta) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float sx[BK][BM + 4];
  __shared__ float sw[BK][BN + 4];
  const int which = blockIdx.z;
  const int b = find_seq(meta.tbase, meta.n, blockIdx.x);
  const int tile = blockIdx.x - meta.tbase[b];
  const int L = meta.len[b];
  const int j0 = tile * BM;
  const int n0 = blockIdx.y * BN;
  const int64_t row0 = meta.start[b];
  const T* xa = a.xa[which];
  const T* xr = a.xr[which];
  const T* w = a.w[which];
  const int d_in = a.D + a.m;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < d_in; k0 += BK) {
    // X tile: 64 rows x 16 k ; thread loads 4 elements
    {
      const int r = threadIdx.x >> 2;          // 0..63
      const int kk = (threadIdx.x & 3) * 4;    // 0,4,8,12
      int j = j0 + r; if (j >= L) j = L - 1;
      const int k = k0 + kk;
      const T* src = (k < a.D) ? xa + (row0 + j) * (int64_t)a.D + k
                               : xr + (row0 + j) * (int64_t)a.m + (k - a.D);
#pragma unroll
      for (int i = 0; i < 4; ++i) sx[kk + i][r] = Elem<T>::to_f32(src[i]);
    }
    // W tile: 16 k x 64 n ; thread loads 4 elements
    {
      const int kk = threadIdx.x >> 4;         // 0..15
      const int nn = (threadIdx.x & 15) * 4;
      const T* src = w + (int64_t)(k0 + kk) * a.d_out + n0 + nn;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        sw[kk][nn + i] = (n0 + nn + i < a.d_out) ? Elem<T>::to_f32(src[i]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float xv[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { xv[i] = sx[kk][ty * 4 + i]; wv[i] = sw[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) acc[i][jn] = fmaf(xv[i], wv[jn], acc[i][jn]);
    }
    __syncthreads();
  }
  const int64_t orow0 = a.rows_from_slots ? (int64_t)meta.sbase[b] * kSlotTokens : 0;
  T* out = a.out[which];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int j = j0 + ty * 4 + i;
    if (j >= L) continue;
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) {
      const int c = n0 + tx * 4 + jn;
      if (c < a.d_out) out[(orow0 + j) * a.ldo + a.col0 + c] = Elem<T>::from_f32(acc[i][jn]);
    }
  }
}

// ---------------------------------------------------------------------------
// Split-K streaming attention over heads that are stored somewhere as rows
// (the target layer's retained heads, or materialised predicted heads):
// scores, online softmax and P.V for GT query heads of one KV head over one
// chunk of `split_tokens` tokens (Eq. 7).  Writes one partial
// (max, sum-exp, unnormalised o) per (chunk, query head).
//   LPR = lanes that share one row = d * sizeof(T) / 16.
// grid.x = chunks (tbase), grid.y = kv heads handled * (G / GT).
// ---------------------------------------------------------------------------
template <typename T>
struct AttnArgs {
  const T* k; const T* v;   // row r, head g at k + r*ld + col0 + g_local*d
  int64_t ld;
  int32_t col0;             // column of the first head handled
  int32_t head0;            // its KV head index (for the query / output head)
  int32_t row_mode;         // 0: row = start[b] + j ; 1: sbase[b]*kSlotTokens + j ; 2: j ;
                            // 3: window rows, row = (seq0 + b) * win.rows() + j, one chunk per sequence
  const T* q;               // [nseq, H_q, d]
  int32_t H_q, G, d;
  float scale;
  int32_t split_tokens;     // multiple of kSlotTokens
  float* part_o;            // [slots, H_q, d]
  float* part_ml;           // [slots, H_q, 2]
  // paper-faithful extras: rotary tables [positions, d/2] (null: none) applied to the key rows by
  // token position; window: modes 0-2 skip the tokens the window holds, mode 3 attends them
  const float* rope_cos = nullptr; const float* rope_sin = nullptr;
  Window win = {0, 0};
  int32_t seq0 = 0;         // mode 3: index of the launch's first sequence in the window buffers
  int32_t win_slot0 = 0;    // mode 3: partial of sequence b goes to slot win_slot0 + b
};

template <typename T, int LPR, int GT>
__global__ __launch_bounds__(256) void attn_split_kernel(AttnArgs<T> a, SeqMeta meta) {
  constexpr int VEC = Elem<T>::kVec;
  constexpr int RPW = 64 / LPR;        // row groups per wave
  constexpr int NRG = 4 * RPW;         // row groups per block
  const int b = find_seq(meta.tbase, meta.n, blockIdx.x);
  const int chunk = blockIdx.x - meta.tbase[b];
  const int L = meta.len[b];
  const int gchunks = a.G / GT;
  const int hl = blockIdx.y / gchunks;           // local kv head
  const int qh0 = (a.head0 + hl) * a.G + (blockIdx.y % gchunks) * GT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rg = wave * RPW + lane / LPR;        // row group in block
  const int li = lane % LPR;                     // lane within row
  const bool wmode = a.row_mode == 3;
  const int64_t row0 = a.row_mode == 0 ? meta.start[b]
                     : a.row_mode == 1 ? (int64_t)meta.sbase[b] * kSlotTokens
                     : wmode ? (int64_t)(a.seq0 + b) * a.win.rows() : 0;
  const int col = a.col0 + hl * a.d + li * VEC;
  // tokens of this chunk: the compressed rows outside the window, or all window rows
  const int jbeg = wmode ? 0 : max(chunk * a.split_tokens, a.win.lo(L));
  const int jend = wmode ? a.win.rows() : min(a.win.hi(L), chunk * a.split_tokens + a.split_tokens);
  const bool rope = a.rope_cos != nullptr;
  const int hc = (li % (LPR / 2)) * VEC;          // this lane's first column in the d/2-wide tables

  float qv[GT][VEC];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    load16<T>(a.q + ((int64_t)b * a.H_q + qh0 + g) * a.d + li * VEC, qv[g]);
#pragma unroll
    for (int i = 0; i < VEC; ++i) qv[g][i] *= a.scale;
  }
  float mx[GT], sm[GT], o[GT][VEC];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    mx[g] = -INFINITY; sm[g] = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) o[g][i] = 0.f;
  }
  constexpr int UN = 4;
  for (int j = jbeg + rg; j < jend; j += NRG * UN) {
    float kv[UN][VEC], vv[UN][VEC];
    int pos[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      int jj = j + u * NRG; if (jj >= jend) jj = jend - 1;
      load16<T>(a.k + (row0 + jj) * a.ld + col, kv[u]);
      load16<T>(a.v + (row0 + jj) * a.ld + col, vv[u]);
      pos[u] = wmode ? a.win.pos_of(jj, L) : jj;
      if (rope) {        // feature i pairs with i + d/2, held by the lane LPR / 2 away
        const int pr = max(pos[u], 0);
        float cs[VEC], sn[VEC];
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
          const float4 c4 = *reinterpret_cast<const float4*>(a.rope_cos + (int64_t)pr * (a.d / 2) + hc + i);
          const float4 s4 = *reinterpret_cast<const float4*>(a.rope_sin + (int64_t)pr * (a.d / 2) + hc + i);
          cs[i] = c4.x; cs[i + 1] = c4.y; cs[i + 2] = c4.z; cs[i + 3] = c4.w;
          sn[i] = s4.x; sn[i + 1] = s4.y; sn[i + 2] = s4.z; sn[i + 3] = s4.w;
        }
        const float sgn = (li < LPR / 2) ? -1.f : 1.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          const float other = __shfl_xor(kv[u][i], LPR / 2, 64);
          kv[u][i] = fmaf(kv[u][i], cs[i], sgn * other * sn[i]);
        }
      }
    }
    // scores of the round's UN rows, then ONE change of the softmax reference per query head and
    // round (one correction factor instead of one per row)
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float sc[UN];
      float mn = mx[g];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const bool live = (j + u * NRG) < jend && pos[u] >= 0;
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) t = fmaf(qv[g][i], kv[u][i], t);
        t = row_sum<LPR>(t);
        sc[u] = live ? t : -INFINITY;
        mn = fmaxf(mn, sc[u]);
      }
      if (mn != -INFINITY) {                       // (uniform over the lanes of a row)
        const float corr = __expf(mx[g] - mn);     // mx = -inf at the start: 0, and o, sm are 0
        float p[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) p[u] = __expf(sc[u] - mn);     // a dead row: exp(-inf) = 0
        sm[g] = sm[g] * corr + ((p[0] + p[1]) + (p[2] + p[3]));
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          float t = o[g][i] * corr;
#pragma unroll
          for (int u = 0; u < UN; ++u) t = fmaf(p[u], vv[u][i], t);
          o[g][i] = t;
        }
        mx[g] = mn;
      }
    }
  }
  // merge the NRG row groups: first inside the wave, then across waves in LDS
  __shared__ float s_m[4][GT], s_l[4][GT];
  __shared__ float s_o[4][GT][LPR * VEC];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    float M = mx[g];
    for (int off = LPR; off < 64; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    const float w = (mx[g] == -INFINITY) ? 0.f : __expf(mx[g] - M);
    float l = sm[g] * w;
    for (int off = LPR; off < 64; off <<= 1) l += __shfl_xor(l, off, 64);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      float x = o[g][i] * w;
      for (int off = LPR; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
      o[g][i] = x;
    }
    if (lane < LPR) {
#pragma unroll
      for (int i = 0; i < VEC; ++i) s_o[wave][g][li * VEC + i] = o[g][i];
    }
    if (lane == 0) { s_m[wave][g] = M; s_l[wave][g] = l; }
  }
  __syncthreads();
  const int slot = wmode ? a.win_slot0 + b : meta.sbase[b] + chunk * (a.split_tokens / kSlotTokens);
  for (int idx = threadIdx.x; idx < GT * a.d; idx += 256) {
    const int g = idx / a.d, c = idx % a.d;
    float M = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
    float l = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float e = (s_m[w][g] == -INFINITY) ? 0.f : __expf(s_m[w][g] - M);
      l += s_l[w][g] * e; acc += s_o[w][g][c] * e;
    }
    const int64_t ph = (int64_t)slot * a.H_q + qh0 + g;
    a.part_o[ph * a.d + c] = acc;
    if (c == 0) { a.part_ml[ph * 2] = M; a.part_ml[ph * 2 + 1] = l; }
  }
}

// ---------------------------------------------------------------------------
// Scores only, over heads stored as rows (the target layer's retained heads):
// S^T[h, slot * 128 + j] = scale * q_h . rot_j(k_j) for GT query heads of one KV
// head over one chunk of tokens; base-2 logits if the caller folds log2(e) into
// the scale.  Same row / lane layout and the same rotary handling as
// attn_split_kernel.  grid.x = chunks (tbase), grid.y = kv heads * (G / GT).
// ---------------------------------------------------------------------------
template <typename T, int LPR, int GT>
__global__ __launch_bounds__(256) void row_scores_kernel(AttnArgs<T> a, float* s_out, int64_t s_ld,
                                                         SeqMeta meta) {
  constexpr int VEC = Elem<T>::kVec;
  constexpr int RPW = 64 / LPR, NRG = 4 * RPW;
  const int b = find_seq(meta.tbase, meta.n, blockIdx.x);
  const int chunk = blockIdx.x - meta.tbase[b];
  const int L = meta.len[b];
  const int gchunks = a.G / GT;
  const int hl = blockIdx.y / gchunks;
  const int qh0 = (a.head0 + hl) * a.G + (blockIdx.y % gchunks) * GT;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rg = wave * RPW + lane / LPR, li = lane % LPR;
  const int64_t row0 = meta.start[b];
  const int col = a.col0 + hl * a.d + li * VEC;
  const int jbeg = chunk * a.split_tokens, jend = min(L, jbeg + a.split_tokens);
  const bool rope = a.rope_cos != nullptr;
  const int hc = (li % (LPR / 2)) * VEC;
  float qv[GT][VEC];
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    load16<T>(a.q + ((int64_t)b * a.H_q + qh0 + g) * a.d + li * VEC, qv[g]);
#pragma unroll
    for (int i = 0; i < VEC; ++i) qv[g][i] *= a.scale;
  }
  float* dst = s_out + (int64_t)qh0 * s_ld + (int64_t)meta.sbase[b] * kSlotTokens;
  constexpr int UN = 4;
  for (int j = jbeg + rg; j < jend; j += NRG * UN) {
    float kv[UN][VEC];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int jj = min(j + u * NRG, jend - 1);
      load16<T>(a.k + (row0 + jj) * a.ld + col, kv[u]);
      if (rope) {
        float cs[VEC], sn[VEC];
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
          const float4 c4 = *reinterpret_cast<const float4*>(a.rope_cos + (int64_t)jj * (a.d / 2) + hc + i);
          const float4 s4 = *reinterpret_cast<const float4*>(a.rope_sin + (int64_t)jj * (a.d / 2) + hc + i);
          cs[i] = c4.x; cs[i + 1] = c4.y; cs[i + 2] = c4.z; cs[i + 3] = c4.w;
          sn[i] = s4.x; sn[i + 1] = s4.y; sn[i + 2] = s4.z; sn[i + 3] = s4.w;
        }
        const float sgn = (li < LPR / 2) ? -1.f : 1.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          const float other = __shfl_xor(kv[u][i], LPR / 2, 64);
          kv[u][i] = fmaf(kv[u][i], cs[i], sgn * other * sn[i]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int jj = j + u * NRG;
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        float sc = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) sc = fmaf(qv[g][i], kv[u][i], sc);
        sc = row_sum<LPR>(sc);
        if (li == 0 && jj < jend) dst[(int64_t)g * s_ld + jj] = sc;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Merge of the split partials of one (sequence, query head): exact
// re-association of the softmax-weighted sum.  Heads below `n_stream_heads`
// (in KV-head units) were written every `stream_step` slots, the others every
// `fused_step` slots.  grid = (H_q, nseq, DS), 256 threads.  DS = 1: a workgroup covers all d
// head dims (4 per thread); DS = 4: a quarter of them (1 per thread), for launches with few
// (sequence, head) pairs and long sequences, where 4 x as many workgroups share the reading.
// Each dim's sum runs over the partials in the same order either way: same bits.
// ---------------------------------------------------------------------------
template <typename TO>
struct MergeArgs {
  const float* part_o; const float* part_ml;
  TO* out; float* lse;      // lse may be null
  int32_t H_q, G, d;
  int32_t n_stream_kv_heads, stream_step, fused_step;
  int64_t out_seq0;         // index of the launch's first sequence in out/lse
  int32_t win_slot0 = -1;   // >= 0: one more partial per sequence (its window tokens) at slot win_slot0 + b
};

template <typename TO, int DS, int NT>       // NT threads: 256, or 1024 where sequences are long
__global__ __launch_bounds__(NT) void merge_kernel(MergeArgs<TO> a, SeqMeta meta) {
  constexpr int EPT = DS == 1 ? 4 : 1;          // head dims per thread
  constexpr int NW = NT / 64, NG = NT / 32;      // waves, groups of 32 threads
  const int h = blockIdx.x, b = blockIdx.y;
  const int dim0 = blockIdx.z * 32;              // DS == 4: this workgroup's 32 dims
  const int step = (h / a.G < a.n_stream_kv_heads) ? a.stream_step : a.fused_step;
  const int nreg = (meta.sbase[b + 1] - meta.sbase[b] + step - 1) / step;   // regular partials of this head
  const int n = nreg + (a.win_slot0 >= 0 ? 1 : 0);
  const int64_t slot0 = meta.sbase[b];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // partial i of this (sequence, head): its row in part_o / part_ml
  auto ph_of = [&](int i) -> int64_t {
    const int64_t slot = i < nreg ? slot0 + (int64_t)i * step : (int64_t)a.win_slot0 + b;
    return slot * a.H_q + h;
  };
  __shared__ float s_red[NW];
  __shared__ float s_w[NT];
  __shared__ float s_acc[NG][128];
  auto block_reduce = [&](float v, bool is_max) -> float {    // fixed order: same bits every run
    v = is_max ? wave_max(v, 64) : wave_sum(v, 64);
    __syncthreads();                // s_red may still be read from the previous reduction
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) r = is_max ? fmaxf(r, s_red[w]) : r + s_red[w];
    return r;
  };
  // 1. global max of the partial maxima (a partial that covers no token has -inf and weight 0;
  //    at least one partial of every sequence covers a token)
  float M = -INFINITY;
  for (int i = tid; i < n; i += NT) M = fmaxf(M, a.part_ml[ph_of(i) * 2]);
  M = block_reduce(M, true);
  // 2. weighted sums, NT partials at a time: weights exp(m_s - M) go to LDS, then the groups of
  //    32 threads add up the weighted o rows with independent, coalesced loads
  const int grp = tid >> 5, q4 = DS == 1 ? (tid & 31) * 4 : dim0 + (tid & 31);
  const bool dim_ok = q4 < a.d;
  float acc[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
  float lsum = 0.f;
  for (int c0 = 0; c0 < n; c0 += NT) {
    const int i = c0 + tid;
    float w = 0.f;
    if (i < n) {
      const int64_t ph = ph_of(i);
      w = __expf(a.part_ml[ph * 2] - M);
      lsum += w * a.part_ml[ph * 2 + 1];
    }
    __syncthreads();            // previous chunk's weights are no longer read
    s_w[tid] = w;
    __syncthreads();
    const int cn = min(NT, n - c0);
    if (dim_ok) {
      // 16 partial rows per round, all loads issued before the first is used (the loop is bound
      // by memory latency, not by volume); rows past the end repeat the last one with weight 0
      constexpr int NB = 16;
      for (int j0 = grp; j0 < cn; j0 += NG * NB) {
        float ov[NB][EPT], wv[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int j = j0 + NG * u;
          const float* src = a.part_o + ph_of(c0 + min(j, cn - 1)) * a.d + q4;
          if constexpr (DS == 1) {
            const float4 o = *reinterpret_cast<const float4*>(src);
            ov[u][0] = o.x; ov[u][1] = o.y; ov[u][2] = o.z; ov[u][3] = o.w;
          } else {
            ov[u][0] = *src;
          }
          wv[u] = j < cn ? s_w[min(j, NT - 1)] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
          for (int e = 0; e < EPT; ++e) acc[e] = fmaf(wv[u], ov[u][e], acc[e]);
      }
    }
  }
  const float ll = block_reduce(lsum, false);
  if (dim_ok) {
#pragma unroll
    for (int e = 0; e < EPT; ++e) s_acc[grp][(DS == 1 ? q4 : (tid & 31)) + e] = acc[e];
  }
  __syncthreads();
  const int nd = DS == 1 ? a.d : min(32, a.d - dim0);
  if (tid < nd) {
    float r = 0.f;
#pragma unroll
    for (int g = 0; g < NG; ++g) r += s_acc[g][tid];
    r /= ll;
    const int64_t oh = (a.out_seq0 + b) * a.H_q + h;
    const int dim = DS == 1 ? tid : dim0 + tid;
    if constexpr (sizeof(TO) == 2) a.out[oh * a.d + dim] = f32_to_bf16(r);
    else a.out[oh * a.d + dim] = r;
    if (dim == 0 && a.lse) a.lse[oh] = M + __logf(ll);
  }
}

}  // namespace echokv
