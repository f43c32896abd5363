// libechokv: C-ABI entry points.  Host side only validates, plans and launches;
// every step of the path runs in the HIP kernels included below.
#include "../../include/echokv.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"
#include "stream_kernels.h"
#include "fused_decode.h"
#include "fused_decode_f32.h"
#include "fused_decode_dma.h"
#include "prefill_kernels.h"
#include "absorbed_decode.h"
#include "fit_kernels.h"

using namespace echokv;

namespace {

struct Dims {
  int H_q, H_kv, d, D, m, d_in, d_out, G, es, oes;
  // m = g0*d + r: g0 whole heads are retained; if r > 0 the next head is split.  The kernels then
  // work on d_out_v = d_out + r "virtual" output columns: the weights are extended by r selector
  // columns that copy the split head's retained dims, so that head looks fully predicted to them.
  int g0, r, d_out_v;
  bool bf16, out_bf16;
  bool w_aug;      // ECHOKV_FLAG_W_AUGMENTED: the caller's weights carry the selector columns already
  float scale;
};

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int check_shape(const echokv_shape* s, Dims* o) {
  if (!s) return ECHOKV_ERR_NULL;
  if (s->dtype != ECHOKV_BF16 && s->dtype != ECHOKV_F32) return ECHOKV_ERR_DTYPE;
  if (s->out_dtype != ECHOKV_BF16 && s->out_dtype != ECHOKV_F32) return ECHOKV_ERR_DTYPE;
  if (s->n_q_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0) return ECHOKV_ERR_SHAPE;
  if (s->n_q_heads % s->n_kv_heads) return ECHOKV_ERR_SHAPE;
  if (s->n_kv_heads > 4096 || s->n_q_heads > 65536) return ECHOKV_ERR_SHAPE;
  const int64_t D = (int64_t)s->n_kv_heads * s->head_dim;
  if (s->n_retained < 0 || s->n_retained > D) return ECHOKV_ERR_SHAPE;
  if (s->head_dim != 64 && s->head_dim != 128) return ECHOKV_ERR_UNSUPPORTED;
  if (s->n_retained % 64) return ECHOKV_ERR_UNSUPPORTED;   // k-tiles of 64 input dims
  if (!std::isfinite(s->softmax_scale)) return ECHOKV_ERR_SHAPE;
  o->H_q = s->n_q_heads; o->H_kv = s->n_kv_heads; o->d = s->head_dim;
  o->D = (int)D; o->m = s->n_retained; o->d_in = o->D + o->m; o->d_out = o->D - o->m;
  o->G = o->H_q / o->H_kv;
  o->g0 = o->m / o->d; o->r = o->m % o->d; o->d_out_v = o->d_out + o->r;
  o->bf16 = s->dtype == ECHOKV_BF16; o->out_bf16 = s->out_dtype == ECHOKV_BF16;
  o->w_aug = (s->flags & ECHOKV_FLAG_W_AUGMENTED) != 0;
  o->es = o->bf16 ? 2 : 4; o->oes = o->out_bf16 ? 2 : 4;
  o->scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / std::sqrt((float)o->d);
  return ECHOKV_OK;
}

int check_cache(const echokv_layer_cache* c, int width) {
  if (!c) return ECHOKV_ERR_NULL;
  if (c->width != width) return ECHOKV_ERR_SHAPE;
  if (c->batch <= 0 || c->pool_tokens <= 0) return ECHOKV_ERR_SHAPE;
  if (!c->seq_start || !c->seq_len || !c->seq_cap) return ECHOKV_ERR_NULL;
  if (width > 0 && (!c->k || !c->v)) return ECHOKV_ERR_NULL;
  for (int b = 0; b < c->batch; ++b) {
    if (c->seq_start[b] < 0 || c->seq_len[b] < 0 || c->seq_cap[b] < c->seq_len[b])
      return ECHOKV_ERR_SHAPE;
    if (c->seq_start[b] + (int64_t)c->seq_cap[b] > c->pool_tokens) return ECHOKV_ERR_SHAPE;
  }
  return ECHOKV_OK;
}

int check_pair(const Dims& dm, const echokv_layer_cache* a, const echokv_layer_cache* t) {
  int rc = check_cache(a, dm.D);
  if (rc) return rc;
  rc = check_cache(t, dm.m);
  if (rc) return rc;
  if (a->batch != t->batch) return ECHOKV_ERR_SHAPE;
  for (int b = 0; b < a->batch; ++b)
    if (a->seq_len[b] != t->seq_len[b]) return ECHOKV_ERR_SHAPE;
  return ECHOKV_OK;
}

inline int slots_for(int64_t tokens) { return (int)((tokens + kSlotTokens - 1) / kSlotTokens); }

// Workspace plan: [extended W_K][extended W_V][partial o][partial (max,sum)][K_hat][V_hat]
struct WsPlan {
  size_t off_po, off_pml, off_kh, off_vh, off_wk, off_wv, total;
};
WsPlan plan_ws(const Dims& dm, int64_t part_slots, int64_t recon_rows) {
  WsPlan p;
  size_t o = 0;
  // extended weights first: their place must not depend on the slot counts of a launch group
  const size_t aug = dm.r ? (size_t)dm.d_in * dm.d_out_v * dm.es : 0;
  p.off_wk = o;  o += align_up(aug);
  p.off_wv = o;  o += align_up(aug);
  p.off_po = o;  o += align_up((size_t)part_slots * dm.H_q * dm.d * 4);
  p.off_pml = o; o += align_up((size_t)part_slots * dm.H_q * 2 * 4);
  p.off_kh = o;  o += align_up((size_t)recon_rows * dm.d_out_v * dm.es);
  p.off_vh = o;  o += align_up((size_t)recon_rows * dm.d_out_v * dm.es);
  p.total = o;
  return p;
}

constexpr int kPrefillQChunk = kMaxSeqPerLaunch;   // queries per launch, streaming prefill

// Fixed scratch of echokv_decode_attn_static: takes the place of the caller's workspace for callers
// that cannot allocate.  Every GPU the library runs on holds its own copy until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels and the planning
// code get the per-device address kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = ECHOKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Device address of this device's copy of `scratch` (looked up once per device).
int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ECHOKV_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ECHOKV_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ECHOKV_OK;
}

// Optional event pairs around the dominant kernels (echokv_profile_*).  Channel 0: the decode
// call's dominant kernel(s); 1: a prefill chunk's predictor product; 2: its attention kernel.
constexpr int kProfChannels = 3;
struct Profiler {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pairs[kProfChannels];   // recorded, not yet read
  std::vector<hipEvent_t> pool;                                          // created once, reused
  bool get(hipEvent_t* e) {
    if (!pool.empty()) { *e = pool.back(); pool.pop_back(); return true; }
    return hipEventCreate(e) == hipSuccess;
  }
};
Profiler g_prof;

// One timed region on a stream.  Does nothing while profiling is off.  Events of a region that is
// left early (an error return between begin and end) go back to the pool.
struct ProfScope {
  int ch = 0;
  hipStream_t st = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  bool open = false;
  int begin(int channel, hipStream_t stream) {
    if (!g_prof.on) return ECHOKV_OK;
    ch = channel; st = stream;
    if (!g_prof.get(&e0)) return ECHOKV_ERR_HIP;
    if (!g_prof.get(&e1)) { g_prof.pool.push_back(e0); return ECHOKV_ERR_HIP; }
    open = true;
    if (hipEventRecord(e0, st) != hipSuccess) return ECHOKV_ERR_HIP;
    return ECHOKV_OK;
  }
  int end() {
    if (!open) return ECHOKV_OK;
    if (hipEventRecord(e1, st) != hipSuccess) return ECHOKV_ERR_HIP;
    g_prof.pairs[ch].emplace_back(e0, e1);
    open = false;
    return ECHOKV_OK;
  }
  ~ProfScope() {
    if (open) { g_prof.pool.push_back(e0); g_prof.pool.push_back(e1); }
  }
};

#define HIP_TRY(expr) do { if ((expr) != hipSuccess) return ECHOKV_ERR_HIP; } while (0)
#define LAUNCH_CHECK() do { if (hipGetLastError() != hipSuccess) return ECHOKV_ERR_HIP; } while (0)

// Fill tbase for a tile size; returns the tile count.
int fill_tiles(SeqMeta& mt, int tile_tokens) {
  int acc = 0;
  for (int b = 0; b < mt.n; ++b) { mt.tbase[b] = acc; acc += (mt.len[b] + tile_tokens - 1) / tile_tokens; }
  mt.tbase[mt.n] = acc;
  return acc;
}
int fill_slots(SeqMeta& mt) {
  int acc = 0;
  for (int b = 0; b < mt.n; ++b) { mt.sbase[b] = acc; acc += slots_for(mt.len[b]); }
  mt.sbase[mt.n] = acc;
  return acc;
}

// Weights as the kernels see them: W itself, or (split head, r > 0) W with r selector columns in
// front, built in the workspace.  Column v < r of the extension copies predictor input
// D + g0*d + v, i.e. retained dim g0*d + v of the target layer, exactly (1 * x in fp32).
template <typename T>
int effective_weights(const Dims& dm, const void* w_k, const void* w_v, char* ws, const WsPlan& wp,
                      const T** wk, const T** wv, hipStream_t st) {
  *wk = (const T*)w_k; *wv = (const T*)w_v;
  if (dm.r == 0 || dm.d_out == 0 || dm.w_aug) return ECHOKV_OK;
  T* ak = (T*)(ws + wp.off_wk);
  T* av = (T*)(ws + wp.off_wv);
  AugArgs<T> a;
  a.w[0] = (const T*)w_k; a.w[1] = (const T*)w_v; a.out[0] = ak; a.out[1] = av;
  a.d_in = dm.d_in; a.d_out = dm.d_out; a.r = dm.r; a.sel0 = dm.D + dm.g0 * dm.d;
  hipLaunchKernelGGL((augment_weights_kernel<T>), dim3(dm.d_in, 2), dim3(256), 0, st, a);
  LAUNCH_CHECK();
  *wk = ak; *wv = av;
  return ECHOKV_OK;
}

template <typename T>
int launch_attn_split(const Dims& dm, AttnArgs<T> a, SeqMeta& mt, int n_kv_heads, hipStream_t st) {
  const int tiles = fill_tiles(mt, a.split_tokens);
  const int GT = (dm.G % 4 == 0) ? 4 : (dm.G % 2 == 0) ? 2 : 1;
  dim3 grid(tiles, n_kv_heads * (dm.G / GT));
  constexpr int LPR64 = 64 * (int)sizeof(T) / 16, LPR128 = 128 * (int)sizeof(T) / 16;
#define ATTN_CASE(LPR_, GT_) \
  hipLaunchKernelGGL((attn_split_kernel<T, LPR_, GT_>), grid, dim3(256), 0, st, a, mt)
  if (dm.d == 64) {
    if (GT == 4) ATTN_CASE(LPR64, 4); else if (GT == 2) ATTN_CASE(LPR64, 2); else ATTN_CASE(LPR64, 1);
  } else {
    if (GT == 4) ATTN_CASE(LPR128, 4); else if (GT == 2) ATTN_CASE(LPR128, 2); else ATTN_CASE(LPR128, 1);
  }
#undef ATTN_CASE
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

// The uncompressed window's tokens: plain attention over its full-width rows, all KV heads,
// one partial per sequence at slot win_slot0 + b of (po, pml).
template <typename T>
int launch_window_attn(const Dims& dm, const echokv_decode_extras* ex, const KvExtras& kx, const T* qq,
                       float* po, float* pml, int b0, int win_slot0, const SeqMeta& mt, hipStream_t st) {
  AttnArgs<T> a;
  a.k = (const T*)ex->win_k; a.v = (const T*)ex->win_v; a.ld = dm.D; a.col0 = 0; a.head0 = 0;
  a.row_mode = 3; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
  a.split_tokens = kSlotTokens;
  a.part_o = po; a.part_ml = pml;
  a.rope_cos = kx.rope_cos; a.rope_sin = kx.rope_sin; a.win = Window{kx.n_sink, kx.n_recent};
  a.seq0 = b0; a.win_slot0 = win_slot0;
  SeqMeta wm = mt;                         // one chunk per sequence
  for (int b = 0; b <= wm.n; ++b) wm.tbase[b] = b;
  const int GT = (dm.G % 4 == 0) ? 4 : (dm.G % 2 == 0) ? 2 : 1;
  dim3 grid(wm.n, dm.H_kv * (dm.G / GT));
  constexpr int LPR64 = 64 * (int)sizeof(T) / 16, LPR128 = 128 * (int)sizeof(T) / 16;
#define WIN_CASE(LPR_, GT_) hipLaunchKernelGGL((attn_split_kernel<T, LPR_, GT_>), grid, dim3(256), 0, st, a, wm)
  if (dm.d == 64) {
    if (GT == 4) WIN_CASE(LPR64, 4); else if (GT == 2) WIN_CASE(LPR64, 2); else WIN_CASE(LPR64, 1);
  } else {
    if (GT == 4) WIN_CASE(LPR128, 4); else if (GT == 2) WIN_CASE(LPR128, 2); else WIN_CASE(LPR128, 1);
  }
#undef WIN_CASE
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

template <typename T>
int launch_recon_fma(const Dims& dm, GemmArgs<T> g, SeqMeta& mt, hipStream_t st) {
  const int tiles = fill_tiles(mt, 64);
  dim3 grid(tiles, (g.d_out + 63) / 64, 2);
  hipLaunchKernelGGL((recon_fma_kernel<T>), grid, dim3(256), 0, st, g, mt);
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

#ifndef ECHOKV_MIN_STREAM_BLOCKS
#define ECHOKV_MIN_STREAM_BLOCKS 2048
#endif
constexpr int kMinStreamBlocks = ECHOKV_MIN_STREAM_BLOCKS;
int pick_split_tokens(int64_t total_tokens, int n_heads_blocks) {
  // enough chunks to fill 256 CUs a few times over, but few partials
  int st = 2048;
  while (st > kSlotTokens && (total_tokens / st) * n_heads_blocks < kMinStreamBlocks) st >>= 1;
  return st;
}

template <typename T, typename TO>
int merge_launch(const Dims& dm, const float* po, const float* pml, void* out, float* lse,
                 int64_t out_seq0, int n_stream, int stream_step, int fused_step, int win_slot0,
                 SeqMeta& mt, hipStream_t st) {
  MergeArgs<TO> ma;
  ma.part_o = po; ma.part_ml = pml; ma.out = (TO*)out; ma.lse = lse;
  ma.H_q = dm.H_q; ma.G = dm.G; ma.d = dm.d;
  ma.n_stream_kv_heads = n_stream; ma.stream_step = stream_step; ma.fused_step = fused_step;
  ma.out_seq0 = out_seq0; ma.win_slot0 = win_slot0;
  // few (sequence, head) pairs with many partials each: four workgroups of 1024 threads per pair,
  // 32 head dims each (the merge is bound by the latency of its reads: more of them in flight)
  int max_slots = 0;
  for (int b = 0; b < mt.n; ++b) max_slots = std::max(max_slots, mt.sbase[b + 1] - mt.sbase[b]);
  if (dm.H_q * mt.n <= 256 && max_slots >= 256)
    hipLaunchKernelGGL((merge_kernel<TO, 4, 1024>), dim3(dm.H_q, mt.n, (dm.d + 31) / 32), dim3(1024), 0, st, ma, mt);
  else
    hipLaunchKernelGGL((merge_kernel<TO, 1, 256>), dim3(dm.H_q, mt.n, 1), dim3(256), 0, st, ma, mt);
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

template <typename T>
int decode_impl(const Dims& dm, uint32_t flags, const echokv_layer_cache* an,
                const echokv_layer_cache* tg, const void* w_k, const void* w_v, const void* q,
                const echokv_decode_extras* ex, void* out, float* lse, char* ws, hipStream_t st) {
  const int n_ret_heads = dm.g0, n_rec_heads = dm.H_kv - n_ret_heads;
  KvExtras kx;
  if (ex) {
    kx.rope_cos = ex->rope_cos; kx.rope_sin = ex->rope_sin;
    if (ex->win_k) { kx.n_sink = ex->n_sink; kx.n_recent = ex->n_recent; }
  }
  const Window win = {kx.n_sink, kx.n_recent};
  const bool fused = !(flags & ECHOKV_FLAG_UNFUSED) && fused_decode_supported<T>(dm.d, dm.G);
  const T* wk = nullptr; const T* wv = nullptr;
  bool have_w = false;
  for (int b0 = 0; b0 < an->batch; b0 += kMaxSeqPerLaunch) {
    SeqMeta mt;
    mt.n = std::min(kMaxSeqPerLaunch, an->batch - b0);
    int64_t tokens = 0;
    for (int b = 0; b < mt.n; ++b) {
      mt.start[b] = an->seq_start[b0 + b]; mt.len[b] = an->seq_len[b0 + b]; tokens += mt.len[b];
    }
    const int slots = fill_slots(mt);
    const WsPlan wp = plan_ws(dm, slots + mt.n, fused ? 0 : (int64_t)slots * kSlotTokens);   // + one window partial per sequence
    if (!have_w) {      // the plan of the first (largest-index-independent) group places the extended weights
      int rcw = effective_weights<T>(dm, w_k, w_v, ws, wp, &wk, &wv, st);
      if (rcw) return rcw;
      have_w = true;
    }
    float* po = (float*)(ws + wp.off_po);
    float* pml = (float*)(ws + wp.off_pml);
    const T* qq = (const T*)q + (int64_t)b0 * dm.H_q * dm.d;
    int stream_step = 1, fused_step = 1;

    if (n_ret_heads > 0) {
      AttnArgs<T> a;
      a.k = (const T*)tg->k; a.v = (const T*)tg->v; a.ld = dm.m; a.col0 = 0; a.head0 = 0;
      a.row_mode = 0; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
      a.split_tokens = pick_split_tokens(tokens, n_ret_heads);
      a.part_o = po; a.part_ml = pml;
      a.rope_cos = kx.rope_cos; a.rope_sin = kx.rope_sin; a.win = win;
      stream_step = a.split_tokens / kSlotTokens;
      int rc = launch_attn_split<T>(dm, a, mt, n_ret_heads, st);
      if (rc) return rc;
    }
    if (n_rec_heads > 0) {
      if (fused) {
        ProfScope prof;
        int rc = prof.begin(0, st);
        if (rc) return rc;
        if constexpr (sizeof(T) == 4)
          rc = launch_fused_decode_f32(dm.H_q, dm.H_kv, dm.d, dm.m, dm.d_out_v, dm.g0, dm.scale,
                                       (const float*)an->k, (const float*)an->v, (const float*)tg->k,
                                       (const float*)tg->v, (const float*)wk, (const float*)wv, qq,
                                       po, pml, mt, &fused_step, st, kx);
        else if ((flags & ECHOKV_FLAG_W_PACKED) && !(flags & ECHOKV_FLAG_STAGED))
          rc = launch_fused_decode_dma(dm.H_q, dm.H_kv, dm.d, dm.m, dm.d_out_v, dm.g0, dm.scale,
                                       (const bf16_t*)an->k, (const bf16_t*)an->v,
                                       (const bf16_t*)tg->k, (const bf16_t*)tg->v,
                                       (const bf16_t*)wk, (const bf16_t*)wv, (const bf16_t*)qq, po,
                                       pml, mt, &fused_step, st, kx);
        else
          rc = launch_fused_decode<T>(dm.H_q, dm.H_kv, dm.d, dm.m, dm.d_out_v, dm.g0, dm.scale,
                                      (const T*)an->k, (const T*)an->v, (const T*)tg->k,
                                      (const T*)tg->v, wk, wv, qq, po,
                                      pml, mt, &fused_step, st, (flags & ECHOKV_FLAG_W_PACKED) != 0, kx);
        if (rc) return rc;
        rc = prof.end();
        if (rc) return rc;
      } else {
        T* kh = (T*)(ws + wp.off_kh);
        T* vh = (T*)(ws + wp.off_vh);
        int rc;
        if (recon_mfma_supported<T>()) {
          rc = launch_recon_mfma<T>(dm.D, dm.m, dm.d_out_v, (const T*)an->k, (const T*)an->v,
                                    (const T*)tg->k, (const T*)tg->v, wk, wv, kh, vh,
                                    dm.d_out_v, 0, mt, st);
        } else {
          GemmArgs<T> g;
          g.xa[0] = (const T*)an->k; g.xa[1] = (const T*)an->v;
          g.xr[0] = (const T*)tg->k; g.xr[1] = (const T*)tg->v;
          g.w[0] = wk; g.w[1] = wv;
          g.out[0] = kh; g.out[1] = vh;
          g.D = dm.D; g.m = dm.m; g.d_out = dm.d_out_v; g.ldo = dm.d_out_v; g.col0 = 0;
          g.rows_from_slots = 1;
          rc = launch_recon_fma<T>(dm, g, mt, st);
        }
        if (rc) return rc;
        AttnArgs<T> a;
        a.k = kh; a.v = vh; a.ld = dm.d_out_v; a.col0 = 0; a.head0 = n_ret_heads;
        a.row_mode = 1; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
        a.split_tokens = pick_split_tokens(tokens, n_rec_heads);
        a.part_o = po; a.part_ml = pml;
        a.rope_cos = kx.rope_cos; a.rope_sin = kx.rope_sin; a.win = win;
        fused_step = a.split_tokens / kSlotTokens;
        rc = launch_attn_split<T>(dm, a, mt, n_rec_heads, st);
        if (rc) return rc;
      }
    }
    int win_slot0 = -1;
    if (win.on()) {
      win_slot0 = slots;                    // placed after the regular slots
      int rcw = launch_window_attn<T>(dm, ex, kx, qq, po, pml, b0, win_slot0, mt, st);
      if (rcw) return rcw;
    }
    int rc = dm.out_bf16
        ? merge_launch<T, bf16_t>(dm, po, pml, out, lse, b0, n_ret_heads, stream_step, fused_step, win_slot0, mt, st)
        : merge_launch<T, float>(dm, po, pml, out, lse, b0, n_ret_heads, stream_step, fused_step, win_slot0, mt, st);
    if (rc) return rc;
  }
  return ECHOKV_OK;
}

template <typename T>
int reconstruct_impl(const Dims& dm, const echokv_layer_cache* an, const echokv_layer_cache* tg,
                     const void* w_k, const void* w_v, int seq, int tok_begin, int tok_end,
                     void* k_out, void* v_out, hipStream_t st) {
  const int64_t rows = tok_end - tok_begin;
  const int64_t row0 = an->seq_start[seq] + tok_begin;
  if (dm.m > 0) {
    Copy2dArgs c;
    c.src[0] = (const char*)tg->k + row0 * dm.m * dm.es;
    c.src[1] = (const char*)tg->v + row0 * dm.m * dm.es;
    c.dst[0] = (char*)k_out; c.dst[1] = (char*)v_out;
    c.src_row_bytes = (int64_t)dm.m * dm.es; c.dst_row_bytes = (int64_t)dm.D * dm.es;
    c.copy_bytes = (int64_t)dm.m * dm.es; c.rows = rows;
    hipLaunchKernelGGL(copy2d_kernel, dim3((unsigned)std::min<int64_t>(rows, 8192), 2), dim3(256), 0, st, c);
    LAUNCH_CHECK();
  }
  if (dm.d_out > 0) {
    SeqMeta mt;
    mt.n = 1; mt.start[0] = row0; mt.len[0] = (int)rows; mt.sbase[0] = 0; mt.sbase[1] = slots_for(rows);
    if (recon_mfma_supported<T>()) {
      // flattened output [retained m ; predicted d_out]: no head alignment involved, plain W
      return launch_recon_mfma<T>(dm.D, dm.m, dm.d_out, (const T*)an->k, (const T*)an->v,
                                  (const T*)tg->k, (const T*)tg->v, (const T*)w_k, (const T*)w_v,
                                  (T*)k_out, (T*)v_out, dm.D, dm.m, mt, st);
    }
    GemmArgs<T> g;
    g.xa[0] = (const T*)an->k; g.xa[1] = (const T*)an->v;
    g.xr[0] = (const T*)tg->k; g.xr[1] = (const T*)tg->v;
    g.w[0] = (const T*)w_k; g.w[1] = (const T*)w_v;
    g.out[0] = (T*)k_out; g.out[1] = (T*)v_out;
    g.D = dm.D; g.m = dm.m; g.d_out = dm.d_out; g.ldo = dm.D; g.col0 = dm.m; g.rows_from_slots = 0;
    return launch_recon_fma<T>(dm, g, mt, st);
  }
  return ECHOKV_OK;
}

// bf16: the MFMA attention kernel keeps its softmax state in registers, so only
// the materialised predicted dims live in the workspace; the fp32 streaming
// path also needs split-K partials for one launch of query rows.
int64_t prefill_part_slots(const Dims& dm, int64_t Ltot, int max_q);
// The MFMA prefill path keeps room for a rotated copy of the retained keys behind the plan.
size_t prefill_krot_offset(const Dims& dm, int64_t Ltot, int max_q) {
  return align_up(plan_ws(dm, prefill_part_slots(dm, Ltot, max_q), (int64_t)slots_for(Ltot) * kSlotTokens).total);
}
int64_t prefill_part_slots(const Dims& dm, int64_t Ltot, int max_q) {
  const bool mfma = dm.bf16 && prefill_mfma_supported<bf16_t>(dm.d);
  return mfma ? 0 : (int64_t)std::min(max_q, kPrefillQChunk) * slots_for(Ltot);
}
// MFMA prefill path: [plan][rotated copy of the retained keys][partials of a launch split over the keys]
size_t prefill_split_offset(const Dims& dm, int64_t Ltot, int max_q) {
  return prefill_krot_offset(dm, Ltot, max_q) + align_up((size_t)Ltot * dm.m * dm.es);
}
// Prefill: predicted dims of the whole visible context are rebuilt once into
// the workspace (every query tile reuses them), then causal attention runs
// over retained heads (from the cache) and predicted heads (from the workspace).
template <typename T>
int prefill_impl(const Dims& dm, const echokv_layer_cache* an, const echokv_layer_cache* tg,
                 const void* w_k, const void* w_v, int seq, const void* q, int T_q, int q_pos0,
                 const float* rope_cos, const float* rope_sin, void* out, float* lse, char* ws,
                 hipStream_t st) {
  const int n_ret_heads = dm.g0, n_rec_heads = dm.H_kv - n_ret_heads;
  const int Ltot = q_pos0 + T_q;
  const int64_t row0 = an->seq_start[seq];
  const WsPlan wp = plan_ws(dm, prefill_part_slots(dm, Ltot, T_q), (int64_t)slots_for(Ltot) * kSlotTokens);
  float* po = (float*)(ws + wp.off_po);
  float* pml = (float*)(ws + wp.off_pml);
  T* kh = (T*)(ws + wp.off_kh);
  T* vh = (T*)(ws + wp.off_vh);
  if (n_rec_heads > 0) {
    const T* wk; const T* wv;
    int rc = effective_weights<T>(dm, w_k, w_v, ws, wp, &wk, &wv, st);
    if (rc) return rc;
    ProfScope prof;
    rc = prof.begin(1, st);
    if (rc) return rc;
    SeqMeta mt;
    mt.n = 1; mt.start[0] = row0; mt.len[0] = Ltot; mt.sbase[0] = 0; mt.sbase[1] = slots_for(Ltot);
    if (recon_mfma_supported<T>()) {
      rc = launch_recon_mfma<T>(dm.D, dm.m, dm.d_out_v, (const T*)an->k, (const T*)an->v,
                                (const T*)tg->k, (const T*)tg->v, wk, wv, kh, vh, dm.d_out_v, 0, mt, st);
      if (rc) return rc;
    } else {
      GemmArgs<T> g;
      g.xa[0] = (const T*)an->k; g.xa[1] = (const T*)an->v;
      g.xr[0] = (const T*)tg->k; g.xr[1] = (const T*)tg->v;
      g.w[0] = wk; g.w[1] = wv;
      g.out[0] = kh; g.out[1] = vh;
      g.D = dm.D; g.m = dm.m; g.d_out = dm.d_out_v; g.ldo = dm.d_out_v; g.col0 = 0; g.rows_from_slots = 0;
      rc = launch_recon_fma<T>(dm, g, mt, st);
      if (rc) return rc;
    }
    rc = prof.end();
    if (rc) return rc;
  }
  if (prefill_mfma_supported<T>(dm.d)) {
    ProfScope prof;
    int rcp = prof.begin(2, st);
    if (rcp) return rcp;
    const T* k_ret = (const T*)tg->k + row0 * dm.m;
    if constexpr (sizeof(T) == 2) {
      if (rope_cos) {
        // rotary embedding: the predicted keys are rotated in place in the workspace, the
        // retained ones into a copy next to them; the attention kernels then run unchanged
        T* krot = (T*)(ws + prefill_krot_offset(dm, Ltot, T_q));
        int rc = launch_rope_rows(kh, dm.d_out_v, kh, dm.d_out_v, n_rec_heads, dm.d, Ltot, rope_cos, rope_sin, st);
        if (rc) return rc;
        rc = launch_rope_rows(k_ret, dm.m, krot, dm.m, n_ret_heads, dm.d, Ltot, rope_cos, rope_sin, st);
        if (rc) return rc;
        if (n_ret_heads > 0) k_ret = krot;
      }
    }
    float* sp_o = (float*)(ws + prefill_split_offset(dm, Ltot, T_q));
    float* sp_ml = sp_o + (size_t)T_q * dm.H_q * prefill_kv_splits(T_q, Ltot, dm.H_q) * dm.d;
    rcp = launch_prefill_mfma<T>(dm.H_q, dm.H_kv, dm.d, dm.m, dm.d_out_v, dm.g0, dm.scale, dm.out_bf16,
                                 k_ret, (const T*)tg->v + row0 * dm.m,
                                 kh, vh, (const T*)q, T_q, q_pos0, out, lse, st, sp_o, sp_ml);
    if (rcp) return rcp;
    return prof.end();
  }
  // streaming path: each query is a virtual sequence of length q_pos0 + i + 1
  for (int i0 = 0; i0 < T_q; i0 += kPrefillQChunk) {
    SeqMeta mt;
    mt.n = std::min(kPrefillQChunk, T_q - i0);
    int64_t tokens = 0;
    for (int i = 0; i < mt.n; ++i) { mt.start[i] = row0; mt.len[i] = q_pos0 + i0 + i + 1; tokens += mt.len[i]; }
    fill_slots(mt);
    const T* qq = (const T*)q + (int64_t)i0 * dm.H_q * dm.d;
    int stream_step = 1, fused_step = 1;
    if (n_ret_heads > 0) {
      AttnArgs<T> a;
      a.k = (const T*)tg->k; a.v = (const T*)tg->v; a.ld = dm.m; a.col0 = 0; a.head0 = 0;
      a.row_mode = 0; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
      a.rope_cos = rope_cos; a.rope_sin = rope_sin;
      a.split_tokens = pick_split_tokens(tokens, n_ret_heads);
      a.part_o = po; a.part_ml = pml;
      stream_step = a.split_tokens / kSlotTokens;
      int rc = launch_attn_split<T>(dm, a, mt, n_ret_heads, st);
      if (rc) return rc;
    }
    if (n_rec_heads > 0) {
      AttnArgs<T> a;
      a.k = kh; a.v = vh; a.ld = dm.d_out_v; a.col0 = 0; a.head0 = n_ret_heads;
      a.row_mode = 2; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
      a.rope_cos = rope_cos; a.rope_sin = rope_sin;
      a.split_tokens = pick_split_tokens(tokens, n_rec_heads);
      a.part_o = po; a.part_ml = pml;
      fused_step = a.split_tokens / kSlotTokens;
      int rc = launch_attn_split<T>(dm, a, mt, n_rec_heads, st);
      if (rc) return rc;
    }
    int rc = dm.out_bf16
        ? merge_launch<T, bf16_t>(dm, po, pml, out, lse, i0, n_ret_heads, stream_step, fused_step, -1, mt, st)
        : merge_launch<T, float>(dm, po, pml, out, lse, i0, n_ret_heads, stream_step, fused_step, -1, mt, st);
    if (rc) return rc;
  }
  return ECHOKV_OK;
}

// ---- one-hidden-layer predictor (Appendix "Prediction Network Architecture") ----------------
// H = act([anchor ; retained] W1) is written to the workspace in bf16 by the MFMA predictor-product
// kernel (activation in its store epilogue); the fused decode kernel then runs on H as its only
// input matrix with W2 as the weights.  Retained heads and the merge are unchanged.
struct MlpPlan { size_t off_po, off_pml, off_hk, off_hv, total; };
MlpPlan plan_mlp(const Dims& dm, int64_t slots, int hidden) {
  MlpPlan p;
  size_t o = 0;
  p.off_po = o;  o += align_up((size_t)slots * dm.H_q * dm.d * 4);
  p.off_pml = o; o += align_up((size_t)slots * dm.H_q * 2 * 4);
  p.off_hk = o;  o += align_up((size_t)slots * kSlotTokens * hidden * 2);
  p.off_hv = o;  o += align_up((size_t)slots * kSlotTokens * hidden * 2);
  p.total = o;
  return p;
}
int check_mlp(const Dims& dm, uint32_t flags, int hidden, int act) {
  if (!dm.bf16 || dm.r != 0 || flags != 0) return ECHOKV_ERR_UNSUPPORTED;
  if (!fused_decode_supported<bf16_t>(dm.d, dm.G)) return ECHOKV_ERR_UNSUPPORTED;
  if (hidden < 64 || hidden % 64 || hidden > (1 << 20)) return ECHOKV_ERR_SHAPE;
  if (act != ECHOKV_ACT_RELU && act != ECHOKV_ACT_SILU) return ECHOKV_ERR_SHAPE;
  return ECHOKV_OK;
}

int mlp_impl(const Dims& dm, const echokv_layer_cache* an, const echokv_layer_cache* tg,
             const bf16_t* w1k, const bf16_t* w2k, const bf16_t* w1v, const bf16_t* w2v, int hidden,
             int act, const bf16_t* q, void* out, float* lse, char* ws, hipStream_t st) {
  typedef bf16_t T;
  const int n_ret_heads = dm.g0, n_rec_heads = dm.H_kv - n_ret_heads;
  for (int b0 = 0; b0 < an->batch; b0 += kMaxSeqPerLaunch) {
    SeqMeta mt;
    mt.n = std::min(kMaxSeqPerLaunch, an->batch - b0);
    int64_t tokens = 0;
    for (int b = 0; b < mt.n; ++b) {
      mt.start[b] = an->seq_start[b0 + b]; mt.len[b] = an->seq_len[b0 + b]; tokens += mt.len[b];
    }
    const int slots = fill_slots(mt);
    const MlpPlan wp = plan_mlp(dm, slots, hidden);
    float* po = (float*)(ws + wp.off_po);
    float* pml = (float*)(ws + wp.off_pml);
    const T* qq = q + (int64_t)b0 * dm.H_q * dm.d;
    int stream_step = 1, fused_step = 1;
    if (n_ret_heads > 0) {
      AttnArgs<T> a;
      a.k = (const T*)tg->k; a.v = (const T*)tg->v; a.ld = dm.m; a.col0 = 0; a.head0 = 0;
      a.row_mode = 0; a.q = qq; a.H_q = dm.H_q; a.G = dm.G; a.d = dm.d; a.scale = dm.scale;
      a.split_tokens = pick_split_tokens(tokens, n_ret_heads);
      a.part_o = po; a.part_ml = pml;
      stream_step = a.split_tokens / kSlotTokens;
      int rc = launch_attn_split<T>(dm, a, mt, n_ret_heads, st);
      if (rc) return rc;
    }
    if (n_rec_heads > 0) {
      ProfScope prof;
      int rc = prof.begin(0, st);
      if (rc) return rc;
      T* hk = (T*)(ws + wp.off_hk);
      T* hv = (T*)(ws + wp.off_hv);
      rc = launch_recon_mfma<T>(dm.D, dm.m, hidden, (const T*)an->k, (const T*)an->v,
                                    (const T*)tg->k, (const T*)tg->v, w1k, w1v, hk, hv, hidden, 0,
                                    mt, st, act);
      if (rc) return rc;
      SeqMeta hm = mt;                       // H rows of sequence b start at its first slot
      for (int b = 0; b < hm.n; ++b) hm.start[b] = (int64_t)mt.sbase[b] * kSlotTokens;
      rc = launch_fused_decode<T>(dm.H_q, dm.H_kv, dm.d, 0, dm.d_out, dm.g0, dm.scale, hk, hv,
                                  (const T*)nullptr, (const T*)nullptr, w2k, w2v, qq, po, pml, hm,
                                  &fused_step, st, false, KvExtras(), hidden);
      if (rc) return rc;
      rc = prof.end();
      if (rc) return rc;
    }
    int rc = dm.out_bf16
        ? merge_launch<T, bf16_t>(dm, po, pml, out, lse, b0, n_ret_heads, stream_step, fused_step, -1, mt, st)
        : merge_launch<T, float>(dm, po, pml, out, lse, b0, n_ret_heads, stream_step, fused_step, -1, mt, st);
    if (rc) return rc;
  }
  return ECHOKV_OK;
}

// ---- weight-absorbed decode: workspace plan and launches ------------------
struct AbsPlan {
  size_t off_u, off_s, off_ml, off_yp, off_y, off_op, off_yml, total;
  int H_pad, n_col_a, n_col_tiles, k_slices, k_slice;
};
inline int abs_col_tiles(int width) { return (width + absorbed::kColTile - 1) / absorbed::kColTile; }
// Tokens per split of the value pass (a multiple of the slot size, at least 1024: the workspace
// bound counts on that).  One workgroup takes one split x one column tile; the chip runs them in
// turns of 256 (one per compute unit), and a workgroup costs its tokens plus a fixed part (the
// reduction over its waves, its partial sums and what the later kernels do per split) worth about
// 700 tokens.  So the time goes like ceil(workgroups / 256) * (split + 700), and the split that
// minimises it is taken: measured over 16 split sizes on configurations 1-3 this model orders
// them as the clock does (configuration 3: 3328 tokens, 240 workgroups, 8 % faster than 1024).
int abs_split_tokens(const Dims& dm, const echokv_layer_cache* an, int b0, int n) {
  const int nct = abs_col_tiles(dm.D) + abs_col_tiles(dm.m);
  int best = 1024;
  int64_t best_cost = -1;
  for (int ts = 1024; ts <= 32768; ts += kSlotTokens) {
    int64_t splits = 0;
    for (int b = 0; b < n; ++b) splits += (an->seq_len[b0 + b] + ts - 1) / ts;
    const int64_t turns = (splits * nct + 255) / 256;
    const int64_t cost = turns * (ts + 700);
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = ts; }
  }
  return best;
}
AbsPlan plan_absorbed(const Dims& dm, int nseq, int64_t slots, int64_t splits) {
  AbsPlan p;
  p.H_pad = (dm.H_q + absorbed::kHB - 1) / absorbed::kHB * absorbed::kHB;
  p.n_col_a = abs_col_tiles(dm.D);
  p.n_col_tiles = p.n_col_a + abs_col_tiles(dm.m);
  p.k_slices = std::max(1, std::min(64, dm.d_in / 256));
  p.k_slice = ((dm.d_in + p.k_slices - 1) / p.k_slices + 63) / 64 * 64;
  p.k_slices = (dm.d_in + p.k_slice - 1) / p.k_slice;
  size_t o = 0;
  p.off_u = o;  o += align_up((size_t)nseq * p.H_pad * dm.d_in * 2);
  p.off_s = o;  o += align_up((size_t)p.H_pad * slots * kSlotTokens * 4);
  p.off_ml = o; o += align_up((size_t)splits * p.H_pad * 2 * 4);
  p.off_yp = o; o += align_up((size_t)splits * p.H_pad * dm.d_in * 4);
  p.off_y = o;  o += align_up((size_t)nseq * dm.H_q * dm.d_in * 4);
  p.off_op = o; o += align_up((size_t)p.k_slices * nseq * dm.H_q * dm.d * 4);
  p.off_yml = o; o += align_up((size_t)nseq * dm.H_q * 2 * 4);
  p.total = o;
  return p;
}
// workspace of the absorbed modes: [extended weights (split head, value-absorbed mode only)]
// [absorbed plan][window partial o, (max, sum)]
size_t abs_pre_bytes(const Dims& dm) { return plan_ws(dm, 0, 0).total; }
size_t abs_win_bytes(const Dims& dm, int nseq) {
  return align_up((size_t)nseq * dm.H_q * dm.d * 4) + align_up((size_t)nseq * dm.H_q * 2 * 4);
}
// upper bound for any launch group of a batch holding total_tokens tokens
size_t absorbed_ws_bytes(const Dims& dm, int batch, int64_t total_tokens) {
  const int n = std::min(batch, kMaxSeqPerLaunch);
  return abs_pre_bytes(dm) + plan_absorbed(dm, n, total_tokens / kSlotTokens + n, total_tokens / 1024 + n).total +
         abs_win_bytes(dm, n);
}
constexpr uint32_t kAbsModes = ECHOKV_FLAG_ABSORBED | ECHOKV_FLAG_ABSORB_V;
bool absorbed_supported(const Dims& dm, uint32_t flags) {
  if (!dm.bf16 || (flags & (ECHOKV_FLAG_UNFUSED | ECHOKV_FLAG_W_PACKED | ECHOKV_FLAG_STAGED | ECHOKV_FLAG_W_AUGMENTED))) return false;
  if ((flags & kAbsModes) == kAbsModes) return false;
  if ((flags & ECHOKV_FLAG_ABSORB_V) && !fused_decode_supported<bf16_t>(dm.d, dm.G)) return false;
  return true;
}

// Fills mt for group [b0, b0 + n) and returns (slots, splits, split_tokens) through the plan inputs.
int absorbed_group(const Dims& dm, const echokv_layer_cache* an, int b0, SeqMeta& mt,
                   int* slots, int* splits, int* split_tokens) {
  mt.n = std::min(kMaxSeqPerLaunch, an->batch - b0);
  int64_t tokens = 0;
  for (int b = 0; b < mt.n; ++b) {
    mt.start[b] = an->seq_start[b0 + b]; mt.len[b] = an->seq_len[b0 + b]; tokens += mt.len[b];
  }
  *slots = fill_slots(mt);
  *split_tokens = abs_split_tokens(dm, an, b0, mt.n);
  *splits = fill_tiles(mt, *split_tokens);
  // 32-bit byte offsets inside the score matrix
  if ((int64_t)*slots * kSlotTokens * 4 * absorbed::kHB >= (int64_t)1 << 31) return ECHOKV_ERR_UNSUPPORTED;
  return ECHOKV_OK;
}

size_t absorbed_need(const Dims& dm, const echokv_layer_cache* an) {
  size_t need = 0;
  for (int b0 = 0; b0 < an->batch; b0 += kMaxSeqPerLaunch) {
    SeqMeta mt; int slots, splits, ts;
    if (absorbed_group(dm, an, b0, mt, &slots, &splits, &ts)) return (size_t)-1;
    need = std::max(need, abs_pre_bytes(dm) + plan_absorbed(dm, mt.n, slots, splits).total + abs_win_bytes(dm, mt.n));
  }
  return need;
}

// value_only: keys go through the fused predictor product (scores written out, rotary embedding
// and window allowed); values are absorbed either way.
int absorbed_impl(const Dims& dm, bool value_only, const echokv_layer_cache* an,
                  const echokv_layer_cache* tg, const void* w_k, const void* w_v, const void* q,
                  const echokv_decode_extras* ex, void* out, float* lse, char* ws0, hipStream_t st) {
  typedef bf16_t T;
  KvExtras kx;
  if (ex) {
    kx.rope_cos = ex->rope_cos; kx.rope_sin = ex->rope_sin;
    if (ex->win_k) { kx.n_sink = ex->n_sink; kx.n_recent = ex->n_recent; }
  }
  const Window win = {kx.n_sink, kx.n_recent};
  const WsPlan pre = plan_ws(dm, 0, 0);
  const T* wk = (const T*)w_k; const T* wv_unused = nullptr;
  if (value_only) {
    int rcw = effective_weights<T>(dm, w_k, w_v, ws0, pre, &wk, &wv_unused, st);
    if (rcw) return rcw;
  }
  char* ws = ws0 + pre.total;
  for (int b0 = 0; b0 < an->batch; b0 += kMaxSeqPerLaunch) {
    SeqMeta mt; int slots, splits, ts;
    int rc = absorbed_group(dm, an, b0, mt, &slots, &splits, &ts);
    if (rc) return rc;
    const AbsPlan pl = plan_absorbed(dm, mt.n, slots, splits);
    float* win_po = (float*)(ws + pl.total);
    float* win_pml = (float*)(ws + pl.total + align_up((size_t)mt.n * dm.H_q * dm.d * 4));
    absorbed::Args a;
    a.xa[0] = (const bf16_t*)an->k; a.xa[1] = (const bf16_t*)an->v;
    a.xr[0] = (const bf16_t*)tg->k; a.xr[1] = (const bf16_t*)tg->v;
    a.w[0] = (const bf16_t*)w_k; a.w[1] = (const bf16_t*)w_v;
    a.q = (const bf16_t*)q + (int64_t)b0 * dm.H_q * dm.d;
    a.u = (bf16_t*)(ws + pl.off_u); a.s = (float*)(ws + pl.off_s); a.ml = (float*)(ws + pl.off_ml);
    a.ypart = (float*)(ws + pl.off_yp); a.y = (float*)(ws + pl.off_y); a.opart = (float*)(ws + pl.off_op);
    a.y_ml = (float*)(ws + pl.off_yml); a.win = win;
    a.win_po = win.on() ? win_po : nullptr; a.win_pml = win_pml;
    a.out = out; a.lse = lse; a.out_seq0 = b0;
    a.D = dm.D; a.m = dm.m; a.d_in = dm.d_in; a.d_out = dm.d_out; a.H_q = dm.H_q; a.H_pad = pl.H_pad;
    a.G = dm.G; a.d = dm.d;
    a.s_ld = slots * kSlotTokens; a.split_tokens = ts; a.n_col_a = pl.n_col_a;
    a.n_col_tiles = pl.n_col_tiles; a.k_slices = pl.k_slices; a.k_slice = pl.k_slice;
    a.qscale = dm.scale * 1.4426950408889634f;
    const int nhb = pl.H_pad / absorbed::kHB;
    const int n = mt.n;

    ProfScope prof;
    rc = prof.begin(0, st);
    if (rc) return rc;
    if (!value_only) {
      const dim3 qg((dm.d_in + 127) / 128, dm.H_kv);
      if (dm.d == 128) hipLaunchKernelGGL((absorbed::absorb_q_kernel<128>), qg, dim3(256), 0, st, a, n);
      else hipLaunchKernelGGL((absorbed::absorb_q_kernel<64>), qg, dim3(256), 0, st, a, n);
      LAUNCH_CHECK();
      // few workgroups: one per compute unit with a deeper pipeline; many: two per compute unit
      if ((int64_t)slots * nhb <= 384) hipLaunchKernelGGL(absorbed::scores_kernel<4>, dim3(slots, nhb), dim3(256), 0, st, a, mt);
      else hipLaunchKernelGGL(absorbed::scores_kernel<2>, dim3(slots, nhb), dim3(256), 0, st, a, mt);
      LAUNCH_CHECK();
    } else {
      // scores of the retained heads straight from the target cache, of the predicted heads from
      // the fused predictor product; both in base-2 units, rotated by token position if asked
      SeqMeta km = mt;
      if (dm.g0 > 0) {
        AttnArgs<T> ra;
        ra.k = (const T*)tg->k; ra.v = nullptr; ra.ld = dm.m; ra.col0 = 0; ra.head0 = 0; ra.row_mode = 0;
        ra.q = a.q; ra.H_q = dm.H_q; ra.G = dm.G; ra.d = dm.d; ra.scale = a.qscale;
        ra.split_tokens = pick_split_tokens((int64_t)slots * kSlotTokens, dm.g0);
        ra.part_o = nullptr; ra.part_ml = nullptr;
        ra.rope_cos = kx.rope_cos; ra.rope_sin = kx.rope_sin;
        const int tiles = fill_tiles(km, ra.split_tokens);
        const int GT = (dm.G % 4 == 0) ? 4 : (dm.G % 2 == 0) ? 2 : 1;
        dim3 grid(tiles, dm.g0 * (dm.G / GT));
        constexpr int LPR64 = 8, LPR128 = 16;
#define RS_CASE(LPR_, GT_) hipLaunchKernelGGL((row_scores_kernel<T, LPR_, GT_>), grid, dim3(256), 0, st, ra, a.s, (int64_t)a.s_ld, km)
        if (dm.d == 64) {
          if (GT == 4) RS_CASE(LPR64, 4); else if (GT == 2) RS_CASE(LPR64, 2); else RS_CASE(LPR64, 1);
        } else {
          if (GT == 4) RS_CASE(LPR128, 4); else if (GT == 2) RS_CASE(LPR128, 2); else RS_CASE(LPR128, 1);
        }
#undef RS_CASE
        LAUNCH_CHECK();
      }
      if (dm.H_kv - dm.g0 > 0) {
        rc = launch_fused_kscores<T>(dm.H_q, dm.H_kv, dm.d, dm.m, dm.d_out_v, dm.g0, a.qscale,
                                     (const T*)an->k, (const T*)tg->k, wk, a.q, a.s, a.s_ld, km, st, kx);
        if (rc) return rc;
      }
      if (win.on()) {       // the window's tokens: one o-space partial per sequence
        rc = launch_window_attn<T>(dm, ex, kx, a.q, win_po, win_pml, b0, 0, mt, st);
        if (rc) return rc;
      }
    }
    // few long pieces: more threads on each
    if ((int64_t)dm.H_q * splits < 1024 && ts >= 2048) hipLaunchKernelGGL(absorbed::softmax_stats_kernel<1024>, dim3(dm.H_q, splits), dim3(1024), 0, st, a, mt);
    else hipLaunchKernelGGL(absorbed::softmax_stats_kernel<256>, dim3(dm.H_q, splits), dim3(256), 0, st, a, mt);
    LAUNCH_CHECK();
    int max_splits = 0;
    for (int b = 0; b < n; ++b) max_splits = std::max(max_splits, mt.tbase[b + 1] - mt.tbase[b]);
    a.single_split = max_splits == 1 ? 1 : 0;
    hipLaunchKernelGGL(absorbed::pv_kernel, dim3(splits * pl.n_col_tiles, nhb), dim3(absorbed::kPvWaves * 64), 0, st, a, mt);
    LAUNCH_CHECK();
    if (max_splits == 1) {
      // (the value pass has written y and its (max, sum) itself)
    } else if (max_splits > 8) hipLaunchKernelGGL(absorbed::y_sum_kernel<4>, dim3((dm.d_in + 255) / 256, dm.H_q, n), dim3(256), 0, st, a, mt);
    else hipLaunchKernelGGL(absorbed::y_sum_kernel<1>, dim3((dm.d_in + 1023) / 1024, dm.H_q, n), dim3(256), 0, st, a, mt);
    LAUNCH_CHECK();
    const dim3 og(dm.H_kv, pl.k_slices, (n * dm.G + 31) / 32);
    if (dm.d == 128) hipLaunchKernelGGL((absorbed::out_partial_kernel<128>), og, dim3(256), 0, st, a, n);
    else hipLaunchKernelGGL((absorbed::out_partial_kernel<64>), og, dim3(256), 0, st, a, n);
    LAUNCH_CHECK();
    const int fb = (int)(((int64_t)n * dm.H_q * dm.d + 255) / 256);
    if (dm.out_bf16) hipLaunchKernelGGL((absorbed::out_final_kernel<bf16_t>), dim3(fb), dim3(256), 0, st, a, n);
    else hipLaunchKernelGGL((absorbed::out_final_kernel<float>), dim3(fb), dim3(256), 0, st, a, n);
    LAUNCH_CHECK();
    rc = prof.end();
    if (rc) return rc;
  }
  return ECHOKV_OK;
}

size_t decode_ws_bytes(const Dims& dm, int batch, int64_t total_tokens, bool unfused) {
  const int64_t slots = total_tokens / kSlotTokens + 2 * (int64_t)batch;   // + one window partial per sequence
  return plan_ws(dm, slots, unfused ? slots * kSlotTokens : 0).total;
}
// MFMA prefill path: [plan][rotated copy of the retained keys][partials of a launch split over the keys]
size_t prefill_ws_bytes(const Dims& dm, int64_t Ltot, int max_q) {
  const bool mfma = dm.bf16 && prefill_mfma_supported<bf16_t>(dm.d);
  if (!mfma) return prefill_krot_offset(dm, Ltot, max_q);
  // the partials of the largest split launch any chunk of up to max_q queries can take: the
  // number of shares only changes where the number of query blocks does
  size_t split = 0;
  // (chunks of kMinQueries queries and more are not split)
  for (int tq : {std::min(max_q, prefill::dma::kMinQueries - 1), prefill::dma::BQ, 2 * prefill::dma::BQ})
    if (tq <= max_q) split = std::max(split, prefill_split_floats(tq, Ltot, dm.H_q, dm.d) * 4);
  return prefill_split_offset(dm, Ltot, max_q) + align_up(split);
}

}  // namespace

extern "C" {

const char* echokv_status_string(int status) {
  switch (status) {
    case ECHOKV_OK: return "ok";
    case ECHOKV_ERR_NULL: return "null pointer";
    case ECHOKV_ERR_SHAPE: return "inconsistent or out-of-range shape";
    case ECHOKV_ERR_DTYPE: return "unknown dtype";
    case ECHOKV_ERR_CAPACITY: return "append exceeds reserved rows";
    case ECHOKV_ERR_WORKSPACE: return "workspace missing or too small";
    case ECHOKV_ERR_UNSUPPORTED: return "configuration not supported by this build";
    case ECHOKV_ERR_HIP: return "HIP runtime error";
    case ECHOKV_ERR_STATIC_LIMIT: return "request needs more than the fixed scratch of echokv_decode_attn_static";
    default: return "unknown status";
  }
}

size_t echokv_workspace_bytes(const echokv_shape* shape, int32_t batch, int64_t total_tokens,
                              int32_t max_q) {
  Dims dm;
  if (check_shape(shape, &dm) != ECHOKV_OK || batch <= 0 || total_tokens <= 0 || max_q < 0) return 0;
  size_t need = decode_ws_bytes(dm, batch, total_tokens, true);
  if ((shape->flags & kAbsModes) && absorbed_supported(dm, shape->flags))
    need = std::max(need, absorbed_ws_bytes(dm, batch, total_tokens));
  if (max_q >= 1) need = std::max(need, prefill_ws_bytes(dm, total_tokens, max_q));
  return need;
}

int echokv_pack_weights(const echokv_shape* shape, const void* w, void* w_packed,
                        void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  if (dm.d_out == 0) return ECHOKV_OK;
  if (!w || !w_packed) return ECHOKV_ERR_NULL;
  if (w == w_packed) return ECHOKV_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  dim3 grid((dm.d_out + 63) / 64, (dm.d_in + 63) / 64);
  if (dm.bf16) hipLaunchKernelGGL((transpose_kernel<bf16_t>), grid, dim3(256), 0, st, (const bf16_t*)w, (bf16_t*)w_packed, dm.d_in, dm.d_out, (int64_t)dm.d_out);
  else hipLaunchKernelGGL((transpose_kernel<float>), grid, dim3(256), 0, st, (const float*)w, (float*)w_packed, dm.d_in, dm.d_out, (int64_t)dm.d_out);
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

size_t echokv_augmented_weight_elems(const echokv_shape* shape) {
  Dims dm;
  if (check_shape(shape, &dm) != ECHOKV_OK) return 0;
  return (size_t)dm.d_in * dm.d_out_v;
}

int echokv_augment_weights(const echokv_shape* shape, const void* w_k, const void* w_v,
                           void* w_k_aug, void* w_v_aug, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  if (dm.d_out == 0) return ECHOKV_OK;
  if (!w_k || !w_v || !w_k_aug || !w_v_aug) return ECHOKV_ERR_NULL;
  if (w_k == w_k_aug || w_v == w_v_aug || w_k_aug == w_v_aug) return ECHOKV_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dm.bf16) {
    AugArgs<bf16_t> a;
    a.w[0] = (const bf16_t*)w_k; a.w[1] = (const bf16_t*)w_v; a.out[0] = (bf16_t*)w_k_aug; a.out[1] = (bf16_t*)w_v_aug;
    a.d_in = dm.d_in; a.d_out = dm.d_out; a.r = dm.r; a.sel0 = dm.D + dm.g0 * dm.d;
    hipLaunchKernelGGL((augment_weights_kernel<bf16_t>), dim3(dm.d_in, 2), dim3(256), 0, st, a);
  } else {
    AugArgs<float> a;
    a.w[0] = (const float*)w_k; a.w[1] = (const float*)w_v; a.out[0] = (float*)w_k_aug; a.out[1] = (float*)w_v_aug;
    a.d_in = dm.d_in; a.d_out = dm.d_out; a.r = dm.r; a.sel0 = dm.D + dm.g0 * dm.d;
    hipLaunchKernelGGL((augment_weights_kernel<float>), dim3(dm.d_in, 2), dim3(256), 0, st, a);
  }
  LAUNCH_CHECK();
  return ECHOKV_OK;
}

int echokv_profile_enable(int on) {
  g_prof.on = on != 0;
  return ECHOKV_OK;
}

int echokv_profile_read_channel(int channel, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return ECHOKV_ERR_NULL;
  if (channel < 0 || channel >= kProfChannels) return ECHOKV_ERR_SHAPE;
  double tot = 0.0;
  int64_t n = 0;
  int rc = ECHOKV_OK;
  for (auto& pr : g_prof.pairs[channel]) {
    float ms = 0.f;
    if (hipEventSynchronize(pr.second) != hipSuccess ||
        hipEventElapsedTime(&ms, pr.first, pr.second) != hipSuccess) rc = ECHOKV_ERR_HIP;
    else { tot += ms; ++n; }
    g_prof.pool.push_back(pr.first); g_prof.pool.push_back(pr.second);
  }
  g_prof.pairs[channel].clear();
  *total_ms = tot; *launches = n;
  return rc;
}

int echokv_profile_read(double* total_ms, int64_t* launches) {
  return echokv_profile_read_channel(0, total_ms, launches);
}

int echokv_profile_stream_read(const void* buf, size_t bytes, int32_t repeats, double* gb_per_s) {
  if (!buf || !gb_per_s) return ECHOKV_ERR_NULL;
  const int blocks = 12288;
  const size_t per_block = (size_t)8 * 256 * 16;              // bytes one loop round of a block covers
  const size_t rounds = bytes / (per_block * blocks);
  if (rounds == 0 || repeats < 1 || (uintptr_t)buf % 16) return ECHOKV_ERR_SHAPE;
  const int64_t n16 = (int64_t)(rounds * per_block / 16);
  hipEvent_t e0, e1;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  float best = 0.f;
  int rc = ECHOKV_OK;
  for (int r = 0; r < repeats + 1 && rc == ECHOKV_OK; ++r) {      // the first pass warms up
    if (hipEventRecord(e0, 0) != hipSuccess) { rc = ECHOKV_ERR_HIP; break; }
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, 0, (const uint4*)buf, n16,
                       (uint32_t*)nullptr);
    float ms = 0.f;
    if (hipGetLastError() != hipSuccess || hipEventRecord(e1, 0) != hipSuccess ||
        hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
      rc = ECHOKV_ERR_HIP;
    else if (r > 0 && (best == 0.f || ms < best)) best = ms;
  }
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  if (rc) return rc;
  *gb_per_s = (double)n16 * 16 * blocks / (best * 1e-3) / 1e9;
  return ECHOKV_OK;
}

int echokv_cache_append(const echokv_shape* shape, echokv_layer_cache* dst, const void* k_new,
                        const void* v_new, const int32_t* n_new, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  if (!dst) return ECHOKV_ERR_NULL;
  if (dst->width != dm.D && dst->width != dm.m) return ECHOKV_ERR_SHAPE;
  rc = check_cache(dst, dst->width);
  if (rc) return rc;
  if (!n_new) return ECHOKV_ERR_NULL;
  int64_t total = 0;
  for (int b = 0; b < dst->batch; ++b) {
    if (n_new[b] < 0) return ECHOKV_ERR_SHAPE;
    if ((int64_t)dst->seq_len[b] + n_new[b] > dst->seq_cap[b]) return ECHOKV_ERR_CAPACITY;
    total += n_new[b];
  }
  if (total > 0 && (!k_new || !v_new)) return ECHOKV_ERR_NULL;
  if (total > INT32_MAX) return ECHOKV_ERR_SHAPE;
  hipStream_t st = (hipStream_t)hip_stream;
  if (dst->width > 0) {
    int64_t done = 0;
    for (int b0 = 0; b0 < dst->batch; b0 += kMaxSeqPerLaunch) {
      SeqMeta mt;
      mt.n = std::min(kMaxSeqPerLaunch, dst->batch - b0);
      int acc = 0;
      for (int b = 0; b < mt.n; ++b) {
        mt.start[b] = dst->seq_start[b0 + b]; mt.len[b] = dst->seq_len[b0 + b];
        mt.tbase[b] = acc; acc += n_new[b0 + b];
      }
      mt.tbase[mt.n] = acc;
      if (acc > 0) {
        CopyArgs c;
        c.src[0] = (const char*)k_new + done * dm.D * dm.es;
        c.src[1] = (const char*)v_new + done * dm.D * dm.es;
        c.dst[0] = (char*)dst->k; c.dst[1] = (char*)dst->v;
        c.src_row_bytes = (int64_t)dm.D * dm.es; c.dst_row_bytes = (int64_t)dst->width * dm.es;
        c.rows = acc;
        hipLaunchKernelGGL(append_rows_kernel, dim3(std::min(acc, 16384), 2), dim3(256), 0, st, c, mt);
        LAUNCH_CHECK();
      }
      done += acc;
    }
  }
  for (int b = 0; b < dst->batch; ++b) dst->seq_len[b] += n_new[b];
  return ECHOKV_OK;
}

// In-place form of echokv_cache_compress for one matrix pair: rows [row_begin, row_end) of the
// pool at `base` narrow from D to m dims where they lie.
static int compress_in_place(const Dims& dm, char* k, char* v, int64_t row_begin, int64_t row_end,
                             hipStream_t st) {
  const int64_t sb = (int64_t)dm.D * dm.es, db = (int64_t)dm.m * dm.es;
  // rows [r0, r1) can move as one plain copy once their destination ends at or below the byte
  // where their source begins: r1 * m <= r0 * D
  auto chunk_end = [&](int64_t r0) { return std::min(row_end, r0 * dm.D / dm.m); };
  int64_t r0 = row_begin;
  int64_t r_seq = r0;
  while (r_seq < row_end && chunk_end(r_seq) - r_seq < 64) ++r_seq;   // too early for plain copies
  if (r_seq > r0) {
    CompactArgs c;
    c.base[0] = k; c.base[1] = v; c.src_row_bytes = sb; c.dst_row_bytes = db; c.r0 = r0; c.r1 = r_seq;
    hipLaunchKernelGGL(compact_rows_seq_kernel, dim3(2), dim3(256), 0, st, c);
    LAUNCH_CHECK();
    r0 = r_seq;
  }
  while (r0 < row_end) {
    const int64_t r1 = chunk_end(r0);
    Copy2dArgs c;
    c.src[0] = k + r0 * sb; c.src[1] = v + r0 * sb;
    c.dst[0] = k + r0 * db; c.dst[1] = v + r0 * db;
    c.src_row_bytes = sb; c.dst_row_bytes = db; c.copy_bytes = db; c.rows = r1 - r0;
    hipLaunchKernelGGL(copy2d_kernel, dim3((unsigned)std::min<int64_t>(r1 - r0, 16384), 2), dim3(256), 0, st, c);
    LAUNCH_CHECK();
    r0 = r1;
  }
  return ECHOKV_OK;
}

int echokv_cache_compress(const echokv_shape* shape, const echokv_layer_cache* full,
                          echokv_layer_cache* dst, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_cache(full, dm.D);
  if (rc) return rc;
  rc = check_cache(dst, dm.m);
  if (rc) return rc;
  if (full->batch != dst->batch) return ECHOKV_ERR_SHAPE;
  for (int b = 0; b < full->batch; ++b)
    if (full->seq_len[b] > dst->seq_cap[b]) return ECHOKV_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)hip_stream;
  // in place: dst describes the same pool at the same addresses, rows narrowed to m dims
  const bool in_place = dm.m > 0 && dst->k == full->k && dst->v == full->v;
  if (dm.m > 0 && !in_place) {
    // any other overlap of the two caches is refused
    auto overlaps = [&](const void* a, int64_t an, const void* b2, int64_t bn) {
      const char* x = (const char*)a; const char* y = (const char*)b2;
      return x < y + bn && y < x + an;
    };
    const int64_t fb = full->pool_tokens * (int64_t)dm.D * dm.es, db = dst->pool_tokens * (int64_t)dm.m * dm.es;
    if (overlaps(full->k, fb, dst->k, db) || overlaps(full->v, fb, dst->v, db) ||
        overlaps(full->k, fb, dst->v, db) || overlaps(full->v, fb, dst->k, db))
      return ECHOKV_ERR_UNSUPPORTED;
  }
  if (in_place) {
    int64_t row_begin = INT64_MAX, row_end = 0;
    for (int b = 0; b < full->batch; ++b) {
      if (dst->seq_start[b] != full->seq_start[b]) return ECHOKV_ERR_UNSUPPORTED;   // same rows, narrower
      if (full->seq_len[b] == 0) continue;
      row_begin = std::min(row_begin, full->seq_start[b]);
      row_end = std::max(row_end, full->seq_start[b] + (int64_t)full->seq_len[b]);
    }
    if (dm.m < dm.D && row_end > row_begin) {
      rc = compress_in_place(dm, (char*)full->k, (char*)full->v, row_begin, row_end, st);
      if (rc) return rc;
    }
  } else if (dm.m > 0) {
    for (int b = 0; b < full->batch; ++b) {
      const int64_t rows = full->seq_len[b];
      if (rows == 0) continue;
      Copy2dArgs c;
      c.src[0] = (const char*)full->k + full->seq_start[b] * dm.D * dm.es;
      c.src[1] = (const char*)full->v + full->seq_start[b] * dm.D * dm.es;
      c.dst[0] = (char*)dst->k + dst->seq_start[b] * dm.m * dm.es;
      c.dst[1] = (char*)dst->v + dst->seq_start[b] * dm.m * dm.es;
      c.src_row_bytes = (int64_t)dm.D * dm.es; c.dst_row_bytes = (int64_t)dm.m * dm.es;
      c.copy_bytes = (int64_t)dm.m * dm.es; c.rows = rows;
      hipLaunchKernelGGL(copy2d_kernel, dim3((unsigned)std::min<int64_t>(rows, 16384), 2), dim3(256), 0, st, c);
      LAUNCH_CHECK();
    }
  }
  for (int b = 0; b < full->batch; ++b) dst->seq_len[b] = full->seq_len[b];
  return ECHOKV_OK;
}

int echokv_reconstruct(const echokv_shape* shape, const echokv_layer_cache* anchor,
                       const echokv_layer_cache* target, const void* w_k, const void* w_v,
                       int32_t seq, int32_t tok_begin, int32_t tok_end, void* k_out, void* v_out,
                       void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_pair(dm, anchor, target);
  if (rc) return rc;
  if (shape->flags & (ECHOKV_FLAG_W_PACKED | ECHOKV_FLAG_W_AUGMENTED)) return ECHOKV_ERR_UNSUPPORTED;
  if (seq < 0 || seq >= anchor->batch) return ECHOKV_ERR_SHAPE;
  if (tok_begin < 0 || tok_end < tok_begin || tok_end > anchor->seq_len[seq]) return ECHOKV_ERR_SHAPE;
  if (dm.d_out > 0 && (!w_k || !w_v)) return ECHOKV_ERR_NULL;
  if (!k_out || !v_out) return ECHOKV_ERR_NULL;
  if (tok_end == tok_begin) return ECHOKV_OK;
  hipStream_t st = (hipStream_t)hip_stream;
  return dm.bf16 ? reconstruct_impl<bf16_t>(dm, anchor, target, w_k, w_v, seq, tok_begin, tok_end, k_out, v_out, st)
                 : reconstruct_impl<float>(dm, anchor, target, w_k, w_v, seq, tok_begin, tok_end, k_out, v_out, st);
}

int echokv_decode_attn_ex(const echokv_shape* shape, const echokv_layer_cache* anchor,
                          const echokv_layer_cache* target, const void* w_k, const void* w_v,
                          const void* q, const echokv_decode_extras* extras, void* out,
                          float* lse_out, void* workspace, size_t workspace_bytes,
                          void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_pair(dm, anchor, target);
  if (rc) return rc;
  if (dm.d_out > 0 && (!w_k || !w_v)) return ECHOKV_ERR_NULL;
  if (!q || !out) return ECHOKV_ERR_NULL;
  int64_t max_chunk_slots = 0;
  int32_t max_len = 0;
  for (int b0 = 0; b0 < anchor->batch; b0 += kMaxSeqPerLaunch) {
    int64_t s = 0;
    const int b1 = std::min(anchor->batch, b0 + kMaxSeqPerLaunch);
    for (int b = b0; b < b1; ++b) {
      if (anchor->seq_len[b] < 1) return ECHOKV_ERR_SHAPE;
      s += slots_for(anchor->seq_len[b]);
      max_len = std::max(max_len, anchor->seq_len[b]);
    }
    max_chunk_slots = std::max(max_chunk_slots, s + (b1 - b0));      // + one window partial per sequence
  }
  bool has_extras = false;
  if (extras) {
    if ((extras->rope_cos == nullptr) != (extras->rope_sin == nullptr)) return ECHOKV_ERR_NULL;
    if ((extras->win_k == nullptr) != (extras->win_v == nullptr)) return ECHOKV_ERR_NULL;
    if (extras->rope_cos && extras->rope_positions < max_len) return ECHOKV_ERR_SHAPE;
    if (extras->win_k && (extras->n_sink < 0 || extras->n_recent < 0 ||
                          extras->n_sink + extras->n_recent < 1)) return ECHOKV_ERR_SHAPE;
    has_extras = extras->rope_cos || extras->win_k;
  }
  if (shape->flags & kAbsModes) {
    if (!absorbed_supported(dm, shape->flags)) return ECHOKV_ERR_UNSUPPORTED;
    // a rotation between reconstruction and the dot product breaks the re-association of the
    // keys: the extras need the value-only mode
    const bool value_only = (shape->flags & ECHOKV_FLAG_ABSORB_V) != 0;
    if (has_extras && !value_only) return ECHOKV_ERR_UNSUPPORTED;
    const size_t need = absorbed_need(dm, anchor);
    if (need == (size_t)-1) return ECHOKV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < need) return ECHOKV_ERR_WORKSPACE;
    if ((uintptr_t)workspace % 256) return ECHOKV_ERR_WORKSPACE;
    return absorbed_impl(dm, value_only, anchor, target, w_k, w_v, q, has_extras ? extras : nullptr, out,
                         lse_out, (char*)workspace, (hipStream_t)hip_stream);
  }
  if ((shape->flags & ECHOKV_FLAG_W_PACKED) &&
      (dm.r != 0 || (shape->flags & ECHOKV_FLAG_UNFUSED) || !dm.bf16 || !fused_decode_supported<bf16_t>(dm.d, dm.G)))
    return ECHOKV_ERR_UNSUPPORTED;
  const bool unfused = (shape->flags & ECHOKV_FLAG_UNFUSED) ||
                       !(dm.bf16 ? fused_decode_supported<bf16_t>(dm.d, dm.G)
                                 : fused_decode_supported<float>(dm.d, dm.G));
  const size_t need = plan_ws(dm, max_chunk_slots, unfused ? max_chunk_slots * kSlotTokens : 0).total;
  if (!workspace || workspace_bytes < need) return ECHOKV_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 256) return ECHOKV_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  const echokv_decode_extras* ex = has_extras ? extras : nullptr;
  return dm.bf16 ? decode_impl<bf16_t>(dm, shape->flags, anchor, target, w_k, w_v, q, ex, out, lse_out, (char*)workspace, st)
                 : decode_impl<float>(dm, shape->flags, anchor, target, w_k, w_v, q, ex, out, lse_out, (char*)workspace, st);
}

int echokv_decode_attn(const echokv_shape* shape, const echokv_layer_cache* anchor,
                       const echokv_layer_cache* target, const void* w_k, const void* w_v,
                       const void* q, void* out, float* lse_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
  return echokv_decode_attn_ex(shape, anchor, target, w_k, w_v, q, nullptr, out, lse_out, workspace,
                               workspace_bytes, hip_stream);
}

int echokv_decode_path(const echokv_shape* shape, int32_t* path_out) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  if (!path_out) return ECHOKV_ERR_NULL;
  const uint32_t f = shape->flags;
  if (f & kAbsModes) {
    if (!absorbed_supported(dm, f)) return ECHOKV_ERR_UNSUPPORTED;
    *path_out = (f & ECHOKV_FLAG_ABSORB_V) ? ECHOKV_PATH_ABSORB_V : ECHOKV_PATH_ABSORBED;
    return ECHOKV_OK;
  }
  const bool can_fuse = dm.bf16 ? fused_decode_supported<bf16_t>(dm.d, dm.G)
                                : fused_decode_supported<float>(dm.d, dm.G);
  if ((f & ECHOKV_FLAG_W_PACKED) && (dm.r != 0 || (f & ECHOKV_FLAG_UNFUSED) || !dm.bf16 || !can_fuse))
    return ECHOKV_ERR_UNSUPPORTED;
  if (dm.d_out == 0) *path_out = ECHOKV_PATH_RETAINED_ONLY;
  else if ((f & ECHOKV_FLAG_UNFUSED) || !can_fuse) *path_out = ECHOKV_PATH_UNFUSED;
  else if ((f & ECHOKV_FLAG_W_PACKED) && !(f & ECHOKV_FLAG_STAGED)) *path_out = ECHOKV_PATH_FUSED_DIRECT;
  else *path_out = ECHOKV_PATH_FUSED;
  return ECHOKV_OK;
}

int echokv_decode_attn_static(const echokv_shape* shape, const echokv_layer_cache* anchor,
                              const echokv_layer_cache* target, const void* w_k, const void* w_v,
                              const void* q, void* out, float* lse_out, void* hip_stream) {
  // argument checks first (a NULL workspace of zero bytes makes the shared path stop right after
  // them, before any HIP call): only a request that is valid but lacks a workspace goes on
  int rc = echokv_decode_attn_ex(shape, anchor, target, w_k, w_v, q, nullptr, out, lse_out, nullptr, 0,
                                 hip_stream);
  if (rc != ECHOKV_ERR_WORKSPACE) return rc;
  void* ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc) return rc;
  rc = echokv_decode_attn_ex(shape, anchor, target, w_k, w_v, q, nullptr, out, lse_out, ptr,
                             kStaticScratchBytes, hip_stream);
  return rc == ECHOKV_ERR_WORKSPACE ? ECHOKV_ERR_STATIC_LIMIT : rc;
}

int echokv_window_append(const echokv_shape* shape, void* win_k, void* win_v, int32_t n_sink,
                         int32_t n_recent, int32_t batch, const int32_t* seq_len_before,
                         const void* k_new, const void* v_new, const int32_t* n_new,
                         void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  if (!win_k || !win_v || !seq_len_before || !n_new) return ECHOKV_ERR_NULL;
  if (batch <= 0 || n_sink < 0 || n_recent < 0 || n_sink + n_recent < 1) return ECHOKV_ERR_SHAPE;
  int64_t total = 0;
  for (int b = 0; b < batch; ++b) {
    if (seq_len_before[b] < 0 || n_new[b] < 0) return ECHOKV_ERR_SHAPE;
    total += n_new[b];
  }
  if (total == 0) return ECHOKV_OK;
  if (!k_new || !v_new) return ECHOKV_ERR_NULL;
  hipStream_t st = (hipStream_t)hip_stream;
  int64_t src_row = 0;
  for (int b0 = 0; b0 < batch; b0 += kMaxSeqPerLaunch) {
    SeqMeta mt;
    mt.n = std::min(kMaxSeqPerLaunch, batch - b0);
    int rows = 0;
    for (int b = 0; b < mt.n; ++b) {
      mt.start[b] = seq_len_before[b0 + b]; mt.len[b] = n_new[b0 + b];
      mt.tbase[b] = rows; rows += n_new[b0 + b];
    }
    mt.tbase[mt.n] = rows;
    if (rows == 0) continue;
    WinAppendArgs a;
    const int64_t rb = (int64_t)dm.D * dm.es;
    a.src[0] = (const char*)k_new + src_row * rb; a.src[1] = (const char*)v_new + src_row * rb;
    a.dst[0] = (char*)win_k; a.dst[1] = (char*)win_v;
    a.row_bytes = rb; a.rows = rows; a.seq0 = b0; a.win = Window{n_sink, n_recent};
    hipLaunchKernelGGL(window_append_kernel, dim3(std::min(rows, 4096), 2), dim3(256), 0, st, a, mt);
    LAUNCH_CHECK();
    src_row += rows;
  }
  return ECHOKV_OK;
}

size_t echokv_mlp_workspace_bytes(const echokv_shape* shape, int32_t batch, int64_t total_tokens,
                                  int32_t hidden) {
  Dims dm;
  if (check_shape(shape, &dm) != ECHOKV_OK || batch <= 0 || total_tokens <= 0) return 0;
  if (check_mlp(dm, shape->flags, hidden, ECHOKV_ACT_RELU) != ECHOKV_OK) return 0;
  return plan_mlp(dm, total_tokens / kSlotTokens + batch, hidden).total;
}

int echokv_decode_attn_mlp(const echokv_shape* shape, const echokv_layer_cache* anchor,
                           const echokv_layer_cache* target, const void* w1_k, const void* w2_k,
                           const void* w1_v, const void* w2_v, int32_t hidden, int32_t activation,
                           const void* q, void* out, float* lse_out, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_pair(dm, anchor, target);
  if (rc) return rc;
  rc = check_mlp(dm, shape->flags, hidden, activation);
  if (rc) return rc;
  if (dm.d_out > 0 && (!w1_k || !w2_k || !w1_v || !w2_v)) return ECHOKV_ERR_NULL;
  if (!q || !out) return ECHOKV_ERR_NULL;
  int64_t max_chunk_slots = 0;
  for (int b0 = 0; b0 < anchor->batch; b0 += kMaxSeqPerLaunch) {
    int64_t s = 0;
    for (int b = b0; b < std::min(anchor->batch, b0 + kMaxSeqPerLaunch); ++b) {
      if (anchor->seq_len[b] < 1) return ECHOKV_ERR_SHAPE;
      s += slots_for(anchor->seq_len[b]);
    }
    max_chunk_slots = std::max(max_chunk_slots, s);
  }
  const size_t need = plan_mlp(dm, max_chunk_slots, hidden).total;
  if (!workspace || workspace_bytes < need) return ECHOKV_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 256) return ECHOKV_ERR_WORKSPACE;
  return mlp_impl(dm, anchor, target, (const bf16_t*)w1_k, (const bf16_t*)w2_k, (const bf16_t*)w1_v,
                  (const bf16_t*)w2_v, hidden, activation, (const bf16_t*)q, out, lse_out,
                  (char*)workspace, (hipStream_t)hip_stream);
}

// ---- closed-form fit of the linear predictor (stage-1 reconstruction loss) -----------------
struct FitPlan { size_t off_xt, off_ga, off_gt, off_g, off_b, off_w, off_r, off_p, off_ap, off_part, total; };
static FitPlan plan_fit(const Dims& dm, int64_t n_rows) {
  FitPlan p;
  size_t o = 0;
  const size_t wn = (size_t)dm.d_in * dm.d_out * 4;
  p.off_xt = o; o += align_up((size_t)dm.d_in * n_rows * 2);
  p.off_ga = o; o += align_up((size_t)dm.d_in * dm.D * 4);
  p.off_gt = o; o += align_up((size_t)dm.d_in * dm.D * 4);
  p.off_g = o;  o += align_up((size_t)dm.d_in * dm.d_in * 4);
  p.off_b = o;  o += align_up(wn);
  p.off_w = o;  o += align_up(wn);
  p.off_r = o;  o += align_up(wn);
  p.off_p = o;  o += align_up(wn);
  p.off_ap = o; o += align_up(wn);
  p.off_part = o; o += align_up((size_t)fit::kDotBlocks * 4);
  p.total = o;
  return p;
}
static int check_fit(const Dims& dm, int64_t n_rows) {
  if (!dm.bf16) return ECHOKV_ERR_UNSUPPORTED;
  if (dm.d_out == 0) return ECHOKV_ERR_SHAPE;
  if (n_rows < 64 || n_rows % 64) return ECHOKV_ERR_SHAPE;
  // the Gram product addresses each [n_rows, D] matrix through one 2 GB buffer window
  if (n_rows * (int64_t)dm.D * 2 >= ((int64_t)1 << 31)) return ECHOKV_ERR_UNSUPPORTED;
  // ... and reads X^T [d_in, n_rows] as the row operand of the predictor-product kernel: its row
  // pitch n_rows * 2 bytes goes through a 24-bit multiply, and a tile of 256 rows (+ one k-tile)
  // through the same 2 GB window
  if (n_rows * 2 >= ((int64_t)1 << 24) || 257 * n_rows * 2 >= ((int64_t)1 << 31)) return ECHOKV_ERR_UNSUPPORTED;
  return ECHOKV_OK;
}

size_t echokv_fit_workspace_bytes(const echokv_shape* shape, int64_t n_rows) {
  Dims dm;
  if (check_shape(shape, &dm) != ECHOKV_OK || check_fit(dm, n_rows) != ECHOKV_OK) return 0;
  return plan_fit(dm, n_rows).total;
}

int echokv_fit_linear(const echokv_shape* shape, const void* anchor_rows, const void* target_rows,
                      int64_t n_rows, float ridge, int32_t max_iters, float tol, void* w_out,
                      void* workspace, size_t workspace_bytes, int32_t* iters_out,
                      float* rel_residual_out, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_fit(dm, n_rows);
  if (rc) return rc;
  if (!anchor_rows || !target_rows || !w_out) return ECHOKV_ERR_NULL;
  if (!(ridge >= 0.f) || max_iters < 1 || !(tol > 0.f)) return ECHOKV_ERR_SHAPE;
  const FitPlan pl = plan_fit(dm, n_rows);
  if (!workspace || workspace_bytes < pl.total || (uintptr_t)workspace % 256) return ECHOKV_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  typedef bf16_t T;
  const T* A = (const T*)anchor_rows; const T* Tt = (const T*)target_rows;
  T* xt = (T*)(ws + pl.off_xt);
  float* ga = (float*)(ws + pl.off_ga); float* gt = (float*)(ws + pl.off_gt);
  float* G = (float*)(ws + pl.off_g); float* B = (float*)(ws + pl.off_b);
  float* W = (float*)(ws + pl.off_w); float* R = (float*)(ws + pl.off_r);
  float* P = (float*)(ws + pl.off_p); float* AP = (float*)(ws + pl.off_ap);
  float* part = (float*)(ws + pl.off_part);
  const int T_rows = (int)n_rows;
  const int64_t wn = (int64_t)dm.d_in * dm.d_out;

  // 1. X^T [d_in, n_rows]: the anchor columns, then the target's first m columns (Eq. 3 order)
  hipLaunchKernelGGL((transpose_kernel<T>), dim3((dm.D + 63) / 64, (T_rows + 63) / 64), dim3(256), 0, st,
                     A, xt, T_rows, dm.D, (int64_t)dm.D);
  LAUNCH_CHECK();
  if (dm.m > 0) {
    hipLaunchKernelGGL((transpose_kernel<T>), dim3((dm.m + 63) / 64, (T_rows + 63) / 64), dim3(256), 0, st,
                       Tt, xt + (int64_t)dm.D * T_rows, T_rows, dm.m, (int64_t)dm.D);
    LAUNCH_CHECK();
  }
  // 2. Gram blocks on MFMA, fp32 out: ga = X^T A, gt = X^T T  (rows of "X" here = predictor inputs,
  //    contraction over the token rows)
  {
    SeqMeta mt;
    mt.n = 1; mt.start[0] = 0; mt.len[0] = dm.d_in;
    fill_slots(mt);
    rc = launch_recon_mfma<T>(T_rows, 0, dm.D, xt, xt, (const T*)nullptr, (const T*)nullptr, A, Tt,
                              (T*)ga, (T*)gt, dm.D, 0, mt, st, 0, true);
    if (rc) return rc;
  }
  // 3. G = [ga | gt[:, :m]] (+ ridge on the diagonal via the operator below), B = gt[:, m:]
  hipLaunchKernelGGL(fit::copy_cols_kernel, dim3(1024), dim3(256), 0, st, G, (int64_t)dm.d_in, 0, ga,
                     (int64_t)dm.D, 0, dm.d_in, dm.D);
  LAUNCH_CHECK();
  if (dm.m > 0) {
    hipLaunchKernelGGL(fit::copy_cols_kernel, dim3(1024), dim3(256), 0, st, G, (int64_t)dm.d_in, dm.D, gt,
                       (int64_t)dm.D, 0, dm.d_in, dm.m);
    LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(fit::copy_cols_kernel, dim3(1024), dim3(256), 0, st, B, (int64_t)dm.d_out, 0, gt,
                     (int64_t)dm.D, dm.m, dm.d_in, dm.d_out);
  LAUNCH_CHECK();
  // 4. conjugate gradients on (G + ridge I) W = B, W0 = 0, all columns sharing one step length
  auto dot = [&](const float* x, const float* y, double* out) -> int {
    hipLaunchKernelGGL(fit::dot_kernel, dim3(fit::kDotBlocks), dim3(256), 0, st, x, y, wn, part);
    if (hipGetLastError() != hipSuccess) return ECHOKV_ERR_HIP;
    std::vector<float> h(fit::kDotBlocks);
    if (hipMemcpyAsync(h.data(), part, fit::kDotBlocks * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) return ECHOKV_ERR_HIP;
    double s = 0.0;
    for (float v : h) s += v;
    *out = s;
    return ECHOKV_OK;
  };
  hipLaunchKernelGGL(fit::fill_kernel, dim3(1024), dim3(256), 0, st, W, 0.f, wn);
  LAUNCH_CHECK();
  HIP_TRY(hipMemcpyAsync(R, B, wn * 4, hipMemcpyDeviceToDevice, st));
  HIP_TRY(hipMemcpyAsync(P, B, wn * 4, hipMemcpyDeviceToDevice, st));
  double rr = 0.0, bb = 0.0;
  rc = dot(R, R, &rr);
  if (rc) return rc;
  bb = rr;
  int it = 0;
  for (; it < max_iters && rr > (double)tol * tol * bb && bb > 0.0; ++it) {
    {   // AP = G P (fp32 tile GEMM), + ridge P
      SeqMeta mt;
      mt.n = 1; mt.start[0] = 0; mt.len[0] = dm.d_in;
      fill_slots(mt);
      GemmArgs<float> g;
      g.xa[0] = g.xa[1] = G; g.xr[0] = g.xr[1] = nullptr; g.w[0] = g.w[1] = P; g.out[0] = g.out[1] = AP;
      g.D = dm.d_in; g.m = 0; g.d_out = dm.d_out; g.ldo = dm.d_out; g.col0 = 0; g.rows_from_slots = 0;
      const int tiles = fill_tiles(mt, 64);
      hipLaunchKernelGGL((recon_fma_kernel<float>), dim3(tiles, (dm.d_out + 63) / 64, 1), dim3(256), 0, st, g, mt);
      LAUNCH_CHECK();
      if (ridge > 0.f) {
        hipLaunchKernelGGL(fit::axpy_kernel, dim3(1024), dim3(256), 0, st, AP, P, ridge, wn);
        LAUNCH_CHECK();
      }
    }
    double pap = 0.0;
    rc = dot(P, AP, &pap);
    if (rc) return rc;
    if (!(pap > 0.0)) break;
    const float alpha = (float)(rr / pap);
    hipLaunchKernelGGL(fit::step_kernel, dim3(1024), dim3(256), 0, st, W, R, P, AP, alpha, wn);
    LAUNCH_CHECK();
    double rr_new = 0.0;
    rc = dot(R, R, &rr_new);
    if (rc) return rc;
    hipLaunchKernelGGL(fit::direction_kernel, dim3(1024), dim3(256), 0, st, P, R, (float)(rr_new / rr), wn);
    LAUNCH_CHECK();
    rr = rr_new;
  }
  hipLaunchKernelGGL(fit::to_bf16_kernel, dim3(1024), dim3(256), 0, st, (bf16_t*)w_out, W, wn);
  LAUNCH_CHECK();
  HIP_TRY(hipStreamSynchronize(st));
  if (iters_out) *iters_out = it;
  if (rel_residual_out) *rel_residual_out = bb > 0.0 ? (float)std::sqrt(rr / bb) : 0.f;
  return ECHOKV_OK;
}

int echokv_prefill_attn_ex(const echokv_shape* shape, const echokv_layer_cache* anchor,
                           const echokv_layer_cache* target, const void* w_k, const void* w_v,
                           int32_t seq, const void* q, int32_t T_q, int32_t q_pos0,
                           const echokv_decode_extras* extras, void* out, float* lse_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  Dims dm;
  int rc = check_shape(shape, &dm);
  if (rc) return rc;
  rc = check_pair(dm, anchor, target);
  if (rc) return rc;
  if (shape->flags & ECHOKV_FLAG_W_PACKED) return ECHOKV_ERR_UNSUPPORTED;
  if (seq < 0 || seq >= anchor->batch) return ECHOKV_ERR_SHAPE;
  if (T_q <= 0 || q_pos0 < 0) return ECHOKV_ERR_SHAPE;
  if ((int64_t)q_pos0 + T_q > anchor->seq_len[seq]) return ECHOKV_ERR_SHAPE;
  if (dm.d_out > 0 && (!w_k || !w_v)) return ECHOKV_ERR_NULL;
  if (!q || !out) return ECHOKV_ERR_NULL;
  const float* rope_cos = nullptr; const float* rope_sin = nullptr;
  if (extras) {
    if ((extras->rope_cos == nullptr) != (extras->rope_sin == nullptr)) return ECHOKV_ERR_NULL;
    // the uncompressed window is a decode-side structure: a prefill chunk reads the compressed cache
    if (extras->win_k || extras->win_v) return ECHOKV_ERR_UNSUPPORTED;
    if (extras->rope_cos && extras->rope_positions < q_pos0 + T_q) return ECHOKV_ERR_SHAPE;
    rope_cos = extras->rope_cos; rope_sin = extras->rope_sin;
  }
  const size_t need = prefill_ws_bytes(dm, (int64_t)q_pos0 + T_q, T_q);
  if (!workspace || workspace_bytes < need) return ECHOKV_ERR_WORKSPACE;
  if ((uintptr_t)workspace % 256) return ECHOKV_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)hip_stream;
  return dm.bf16 ? prefill_impl<bf16_t>(dm, anchor, target, w_k, w_v, seq, q, T_q, q_pos0, rope_cos, rope_sin, out, lse_out, (char*)workspace, st)
                 : prefill_impl<float>(dm, anchor, target, w_k, w_v, seq, q, T_q, q_pos0, rope_cos, rope_sin, out, lse_out, (char*)workspace, st);
}

int echokv_prefill_attn(const echokv_shape* shape, const echokv_layer_cache* anchor,
                        const echokv_layer_cache* target, const void* w_k, const void* w_v,
                        int32_t seq, const void* q, int32_t T_q, int32_t q_pos0, void* out,
                        float* lse_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return echokv_prefill_attn_ex(shape, anchor, target, w_k, w_v, seq, q, T_q, q_pos0, nullptr, out,
                                lse_out, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
