/* echokv.h -- C ABI of libechokv: EchoKV attention over a compressed KV cache
 * on AMD MI355X (gfx950).
 *
 * The method (paper Sec. "Network Architecture"): layers are grouped; the first
 * layer of a group (the ANCHOR) keeps its full flattened K/V of width
 * D = H_kv * d (Eq. 1); every other layer of the group (a TARGET) keeps only
 * the first m flattened dims (Eq. 2) and the dropped dims [m, D) are predicted
 * per token by a linear map from [anchor row ; retained row] (Eq. 3, Eq. 4).
 * Attention then runs over [retained ; predicted] reshaped to heads (Eq. 6,
 * Eq. 7).  The predicted dims are recomputed at every use and never stored.
 *
 * Conventions
 *  - Plain C, no exceptions; every entry point returns an echokv_status.
 *  - "device" pointers are HIP device memory on the current device; "HOST"
 *    pointers are ordinary host memory read (or, for seq_len in
 *    echokv_cache_append, written) during the call only.
 *  - The library allocates no device memory and frees none.  Cache, weights,
 *    queries, outputs and workspace are owned by the caller (the one fixed
 *    buffer inside the library's device image belongs to
 *    echokv_decode_attn_static, see there).
 *  - All argument checks run before the first HIP call and leave every buffer
 *    and every host array untouched on failure.
 *  - Work is enqueued on `hip_stream` (a hipStream_t, NULL = default stream);
 *    results are valid once that stream has been synchronised.  Two calls that
 *    share a workspace must be ordered on one stream.
 *  - Threads: calls from several host threads are fine as long as they share no
 *    workspace (or order their use of it) -- the library keeps no state per call.
 *    Exceptions: the first launch of the long-chunk prefill kernels on a device
 *    sets a kernel attribute through an unguarded per-device flag (make the first
 *    echokv_prefill_attn call of a process from one thread), the profiling aids
 *    at the end of this header, and echokv_decode_attn_static.
 *  - Flattening is head-major: flattened dim g*d + i is feature i of KV head g.
 *    Query head h reads KV head h / (H_q / H_kv).
 *  - Row-major everywhere; a "row" is one token.
 */
#ifndef ECHOKV_H
#define ECHOKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ECHOKV_OK = 0,
  ECHOKV_ERR_NULL = 1,        /* a required pointer is NULL */
  ECHOKV_ERR_SHAPE = 2,       /* inconsistent or out-of-range sizes */
  ECHOKV_ERR_DTYPE = 3,       /* unknown dtype code */
  ECHOKV_ERR_CAPACITY = 4,    /* append past a sequence's reserved rows */
  ECHOKV_ERR_WORKSPACE = 5,   /* workspace missing or too small */
  ECHOKV_ERR_UNSUPPORTED = 6, /* legal in the method, not built (e.g. m % 64 != 0) */
  ECHOKV_ERR_HIP = 7,         /* a HIP runtime call or launch failed */
  ECHOKV_ERR_STATIC_LIMIT = 8 /* echokv_decode_attn_static: the request needs more than
                                 ECHOKV_STATIC_SCRATCH_BYTES of scratch */
} echokv_status;

typedef enum { ECHOKV_BF16 = 0, ECHOKV_F32 = 1 } echokv_dtype;

/* flags for echokv_shape.flags */
#define ECHOKV_FLAG_UNFUSED 1u /* decode: materialise the predicted dims in the
                                  workspace, then attend (comparison path) */
#define ECHOKV_FLAG_W_PACKED 2u /* w_k / w_v point at weights laid out by
                                  echokv_pack_weights ([D - m, D + m]); honoured by
                                  echokv_decode_attn on the fused bf16 path, every
                                  other use returns ECHOKV_ERR_UNSUPPORTED */
#define ECHOKV_FLAG_STAGED 4u  /* with W_PACKED: use the register-staged main loop
                                  instead of the direct-to-LDS one (comparison) */
#define ECHOKV_FLAG_ABSORBED 8u /* decode: same output in the other association order
                                  (Eq. 3 is linear): queries are folded into W_K and
                                  the probability-weighted sum of predictor inputs is
                                  multiplied by W_V afterwards, so K-hat / V-hat are
                                  never formed and every cache row is read once.
                                  bf16 caches, row-major weights only; include the
                                  flag in the shape passed to echokv_workspace_bytes */
#define ECHOKV_FLAG_ABSORB_V 16u /* decode: absorb the value side only.  Keys are rebuilt
                                  by the fused predictor product and turned into scores
                                  (so a rotary embedding and the uncompressed window of
                                  echokv_decode_attn_ex stay available); the weighted sum
                                  of predictor inputs is multiplied by W_V afterwards,
                                  which halves the matrix work.  Same conditions as
                                  ECHOKV_FLAG_ABSORBED; the two exclude each other */
#define ECHOKV_FLAG_W_AUGMENTED 32u /* w_k / w_v point at weights extended once by
                                  echokv_augment_weights.  Only a layer whose m splits
                                  a head (m % d != 0, e.g. the paper's m = 64 with
                                  d = 128) has such an extension; without the flag every
                                  decode / prefill call builds it in its workspace.
                                  Honoured by echokv_decode_attn(_ex, _static) and
                                  echokv_prefill_attn(_ex) on the fused and unfused
                                  paths; with an absorbed mode, and in every other
                                  entry point that takes weights,
                                  ECHOKV_ERR_UNSUPPORTED */

/* One (anchor, target) layer pair. */
typedef struct {
  int32_t n_q_heads;   /* H_q */
  int32_t n_kv_heads;  /* H_kv; H_q % H_kv == 0 */
  int32_t head_dim;    /* d; 64 or 128 */
  int32_t n_retained;  /* m, flattened dims the target keeps; 0 <= m <= D, m % 64 == 0
                          (the prefix may end inside a head, as in the paper's m = 64 preset) */
  int32_t dtype;       /* echokv_dtype of cache, weights and queries */
  int32_t out_dtype;   /* echokv_dtype of `out`; accumulation is always fp32 */
  float softmax_scale; /* <= 0 selects 1/sqrt(d) (Appendix "Analysis of QK-KL
                          Divergence Loss", softmax(QK^T/sqrt(d))) */
  uint32_t flags;      /* ECHOKV_FLAG_* */
} echokv_shape;

/* One layer's K and V cache: a token-major pool shared by `batch` sequences.
 * Sequence b owns rows [seq_start[b], seq_start[b] + seq_cap[b]) of which the
 * first seq_len[b] are valid.  width == D for an anchor layer (Eq. 1) and
 * width == m for a target layer (Eq. 2). */
typedef struct {
  void *k;                  /* device [pool_tokens, width] */
  void *v;                  /* device [pool_tokens, width] */
  int32_t width;
  int32_t batch;
  int64_t pool_tokens;
  const int64_t *seq_start; /* HOST [batch] */
  int32_t *seq_len;         /* HOST [batch]; echokv_cache_append adds n_new */
  const int32_t *seq_cap;   /* HOST [batch] */
} echokv_layer_cache;

/* Text for a status code (static storage, never NULL). */
const char *echokv_status_string(int status);

/* Write new tokens into one layer's cache (Eq. 1 for an anchor, Eq. 2 for a
 * target; dropping at write time as in Sec. "Throughput Analysis").
 *   k_new, v_new : device [sum_b n_new[b], D], full width, rows packed by
 *                  sequence in batch order; columns [dst->width, D) are read
 *                  by nobody and stored nowhere.
 *   n_new        : HOST [batch], tokens to add to each sequence (0 allowed).
 * On success seq_len[b] += n_new[b].  ERR_CAPACITY if any sequence would pass
 * seq_cap[b]; nothing is written in that case. */
int echokv_cache_append(const echokv_shape *shape, echokv_layer_cache *dst,
                        const void *k_new, const void *v_new,
                        const int32_t *n_new, void *hip_stream);

/* Switch a target layer from full caching to compressed caching (the on-demand
 * transition of Sec. "Overview of EchoKV": when memory runs short, the dims
 * [m, D) of the layer are evicted and from then on predicted; Eq. 2 says what
 * stays).  Copies the first m dims of every valid row of `full` (width D) into
 * `dst` (width m) and sets dst->seq_len[b] = full->seq_len[b].
 *  - Two buffers: the two caches describe the same sequences but may place them
 *    differently (seq_start, seq_cap); they must not overlap.  The caller frees
 *    the full cache once the stream has passed this call.
 *  - In place (no second buffer, for the moment memory is short): dst->k ==
 *    full->k and dst->v == full->v, dst->seq_start[b] == full->seq_start[b].
 *    The pool [pool_tokens, D] becomes the pool [pool_tokens, m] at the same
 *    address: row r moves from byte offset r * D * es to r * m * es.  Rows
 *    between the first and the last valid row are all moved (gap rows too).
 *    Afterwards the bytes behind pool_tokens * m * es are the caller's to give
 *    back; `full` no longer describes anything.  Any other overlap of the two
 *    caches returns ECHOKV_ERR_UNSUPPORTED.
 * ERR_CAPACITY if a sequence does not fit dst->seq_cap. */
int echokv_cache_compress(const echokv_shape *shape, const echokv_layer_cache *full,
                          echokv_layer_cache *dst, void *hip_stream);

/* Rebuild the full-width K and V rows of tokens [tok_begin, tok_end) of
 * sequence `seq` (Eq. 3 then Eq. 6): out row = [retained m dims ; [anchor row ;
 * retained row] W].
 *   w_k, w_v     : device [D + m, D - m] row-major, no bias; may be NULL iff m == D.
 *   k_out, v_out : device [tok_end - tok_begin, D] in shape->dtype. */
int echokv_reconstruct(const echokv_shape *shape, const echokv_layer_cache *anchor,
                       const echokv_layer_cache *target, const void *w_k,
                       const void *w_v, int32_t seq, int32_t tok_begin,
                       int32_t tok_end, void *k_out, void *v_out, void *hip_stream);

/* One-time re-layout of a predictor weight matrix (Eq. 3) for the decode
 * kernel: w_packed[c, k] = w[k, c], i.e. [D - m, D + m] row-major, each output
 * column's input dims contiguous.  The weights of a layer are constant while
 * serving, so a caller packs them once at load time and passes the packed
 * pointers with ECHOKV_FLAG_W_PACKED set.
 *   w        : device [D + m, D - m] row-major
 *   w_packed : device [D - m, D + m], same dtype, must not overlap w */
int echokv_pack_weights(const echokv_shape *shape, const void *w, void *w_packed,
                        void *hip_stream);

/* One-time extension of the predictor weights of a layer whose retained width
 * splits a head (Eq. 2 with m % d = r > 0; Eq. 6 puts the r retained dims of that
 * head in front of its predicted ones).  The kernels treat the split head as
 * fully predicted: w_aug = [S | w] with r selector columns S in front, column v
 * of S being 1 at input row D + (m - r) + v (that retained dim of the target
 * layer) and 0 elsewhere, so the product copies those dims exactly.  The
 * weights of a layer are constant while serving: extend them once at load time
 * and pass the extended pointers with ECHOKV_FLAG_W_AUGMENTED set.
 *   w_k, w_v         : device [D + m, D - m] row-major
 *   w_k_aug, w_v_aug : device [D + m, D - m + r], same dtype, four distinct buffers
 * With r == 0 the extension is a plain copy (and the flag changes nothing).
 * echokv_augmented_weight_elems: elements of one extended matrix, 0 on a bad shape. */
size_t echokv_augmented_weight_elems(const echokv_shape *shape);
int echokv_augment_weights(const echokv_shape *shape, const void *w_k, const void *w_v,
                           void *w_k_aug, void *w_v_aug, void *hip_stream);

/* Bytes of workspace that echokv_decode_attn (batch sequences holding
 * total_tokens cached tokens in all) needs and, when max_q >= 1, that
 * echokv_prefill_attn needs for chunks of up to max_q queries of one sequence
 * whose visible context (q_pos0 + T_q) is at most total_tokens.  max_q == 0:
 * decode only.  The prefill part holds the predicted dims of the whole visible
 * context (2 (D - m) values per token), a rotated copy of the retained keys,
 * and, for chunks under 1024 queries in front of a long context, the fp32
 * partial results of the launch split over the keys (at most 8 shares of
 * d + 2 words per query and head).  Returns 0 on a bad shape. */
size_t echokv_workspace_bytes(const echokv_shape *shape, int32_t batch,
                              int64_t total_tokens, int32_t max_q);

/* Decode step for the target layer (Eq. 7 with one query per sequence):
 * out[b, h, :] = softmax_j(scale * q[b,h,:] . Kt[b,j,h/G,:]) Vt[b,j,h/G,:]
 * over the seq_len[b] cached tokens, where Kt/Vt heads below m/d are read
 * from the target cache and the others are predicted on the fly (Eq. 3, 6).
 *   q       : device [batch, H_q, d]
 *   out     : device [batch, H_q, d] in shape->out_dtype
 *   lse_out : device [batch, H_q] fp32 log-sum-exp of the scaled scores, or NULL
 * anchor and target must describe the same sequences (equal batch, seq_len).
 * Every seq_len[b] must be >= 1. */
int echokv_decode_attn(const echokv_shape *shape, const echokv_layer_cache *anchor,
                       const echokv_layer_cache *target, const void *w_k,
                       const void *w_v, const void *q, void *out, float *lse_out,
                       void *workspace, size_t workspace_bytes, void *hip_stream);

/* Which kernels echokv_decode_attn will run for `shape` (its flags included),
 * so that a caller can tell beforehand when a layer does not take the fused
 * reconstruct-then-attend kernel.  The fused kernel keeps the softmax
 * numerators of every (KV head in its 128-column wave tile, query head of the
 * group) pair in LDS, at most 8 pairs: (128 / d) * G <= 8.  A layer beyond that
 * (e.g. d = 128 with 16 query heads per KV head) is served by the materialising
 * path -- predictor product into the workspace, then streaming attention --
 * exactly as if ECHOKV_FLAG_UNFUSED were set, and echokv_workspace_bytes
 * already accounts for it.  The same call reports the choice made for the
 * other flags.  *path_out is one of ECHOKV_PATH_*. */
#define ECHOKV_PATH_FUSED 0          /* fused predictor product + attention, row-major W */
#define ECHOKV_PATH_FUSED_DIRECT 1   /* the same with packed W, operands straight into LDS */
#define ECHOKV_PATH_UNFUSED 2        /* K-hat / V-hat materialised in the workspace, then attended */
#define ECHOKV_PATH_ABSORBED 3       /* ECHOKV_FLAG_ABSORBED */
#define ECHOKV_PATH_ABSORB_V 4       /* ECHOKV_FLAG_ABSORB_V */
#define ECHOKV_PATH_RETAINED_ONLY 5  /* m == D: nothing to predict, plain streaming attention */
int echokv_decode_path(const echokv_shape *shape, int32_t *path_out);

/* echokv_decode_attn for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same result as
 * echokv_decode_attn (shape->flags honoured alike), but the split partials (and
 * whatever else the chosen path keeps in its workspace) live in a fixed buffer
 * of ECHOKV_STATIC_SCRATCH_BYTES inside the library's device image instead of a
 * caller-owned workspace.  The call allocates and frees nothing.
 *  - Limit: a request whose echokv_workspace_bytes-style need exceeds
 *    ECHOKV_STATIC_SCRATCH_BYTES returns ECHOKV_ERR_STATIC_LIMIT and touches
 *    nothing.  On the fused path the need is about (tokens / 128 + 2 * batch) *
 *    H_q * (d + 2) * 4 bytes: 32 MiB covers ~250 K cached tokens at H_q = 32,
 *    d = 128.
 *  - Every GPU the library runs on holds one such buffer until the process
 *    ends; all calls on a GPU share it.  It keeps the previous call's contents;
 *    nothing in it needs to start at zero (every partial that is read has been
 *    written by the same call).  Two calls that overlap in time on one GPU
 *    (different streams, different threads) race on it: order them. */
#define ECHOKV_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int echokv_decode_attn_static(const echokv_shape *shape, const echokv_layer_cache *anchor,
                              const echokv_layer_cache *target, const void *w_k,
                              const void *w_v, const void *q, void *out, float *lse_out,
                              void *hip_stream);

/* What the paper's own inference adds around Eq. 7 (both optional, independent):
 *
 * Rotary embedding (Sec. "Network Architecture": the predictor is fed keys taken
 * BEFORE the rotary embedding, so the caches of both layers hold pre-rotation
 * keys).  With rope_cos / rope_sin set, the key of cached token j -- retained or
 * predicted -- is rotated to position j just before the dot product:
 *   k'_i = k_i cos[j, i] - k_{i+d/2} sin[j, i],  k'_{i+d/2} = k_{i+d/2} cos[j, i] + k_i sin[j, i]
 * for i < d/2 in every head (feature i pairs with i + d/2).  q must come in
 * already rotated to its own position.  The tables are the caller's:
 *   rope_cos, rope_sin : device [rope_positions, d/2] fp32; rope_positions >= every seq_len.
 *
 * Uncompressed window (Sec. "Experimental Setting", paragraph "Implement details":
 * the paper exempts the first 4 and the most recent 128 tokens from compression).  With win_k / win_v set, the first
 * n_sink and the latest n_recent positions of every sequence take their keys
 * and values from these full-width rows of the TARGET layer instead of the
 * compressed cache; all other positions are rebuilt as usual.
 *   win_k, win_v : device [batch, n_sink + n_recent, D], dtype of the caches,
 *                  pre-rotation; position p of sequence b is row p if p < n_sink,
 *                  else row n_sink + (p - n_sink) % n_recent (a ring).
 * echokv_window_append keeps the rows current; the compressed cache still
 * receives every token (echokv_cache_append), the window is an extra copy. */
typedef struct {
  const float *rope_cos;
  const float *rope_sin;
  int32_t rope_positions;
  int32_t n_sink;
  int32_t n_recent;
  const void *win_k;
  const void *win_v;
} echokv_decode_extras;

/* echokv_decode_attn with the extras above (extras == NULL, or all of its
 * pointers NULL: the same as echokv_decode_attn).  Not available with
 * ECHOKV_FLAG_ABSORBED (ECHOKV_ERR_UNSUPPORTED); available with
 * ECHOKV_FLAG_ABSORB_V.  Same workspace size. */
int echokv_decode_attn_ex(const echokv_shape *shape, const echokv_layer_cache *anchor,
                          const echokv_layer_cache *target, const void *w_k,
                          const void *w_v, const void *q,
                          const echokv_decode_extras *extras, void *out, float *lse_out,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* Append the full-width rows of new tokens of the target layer to the window.
 *   seq_len_before : HOST [batch] tokens each sequence held before this append
 *   k_new, v_new   : device [sum n_new, D] packed by sequence (the same rows that
 *                    echokv_cache_append is given for the target layer)
 *   n_new          : HOST [batch]
 * Rows that are outside the window once the call's tokens are all in are skipped;
 * the ring row of a token that leaves the local window is overwritten. */
int echokv_window_append(const echokv_shape *shape, void *win_k, void *win_v,
                         int32_t n_sink, int32_t n_recent, int32_t batch,
                         const int32_t *seq_len_before, const void *k_new,
                         const void *v_new, const int32_t *n_new, void *hip_stream);

/* Decode with the one-hidden-layer predictor of Appendix "Prediction Network
 * Architecture" in place of the linear one:
 *   C_hat = act([C_global ; C_local] W1) W2        (Eq. 3 with two layers, bias-free)
 * for keys (w1_k, w2_k) and values (w1_v, w2_v); everything else as
 * echokv_decode_attn.  The paper evaluates a parameter-matched hidden width and
 * hidden = D + m; it names no activation: ECHOKV_ACT_RELU and ECHOKV_ACT_SILU
 * are offered.
 *   w1_* : device [D + m, hidden] row-major;  w2_* : device [hidden, D - m] row-major
 *   hidden : multiple of 64
 * bf16 caches only, m a multiple of the head dim, shape->flags == 0; otherwise
 * ECHOKV_ERR_UNSUPPORTED.  The hidden activations are rounded to bf16 between
 * the layers (they are the second layer's MFMA operand).  Workspace:
 * echokv_mlp_workspace_bytes (it holds the hidden activations of all cached
 * tokens, 2 * hidden * 2 bytes per token, and the split partials). */
#define ECHOKV_ACT_RELU 1
#define ECHOKV_ACT_SILU 2
size_t echokv_mlp_workspace_bytes(const echokv_shape *shape, int32_t batch,
                                  int64_t total_tokens, int32_t hidden);
int echokv_decode_attn_mlp(const echokv_shape *shape, const echokv_layer_cache *anchor,
                           const echokv_layer_cache *target, const void *w1_k,
                           const void *w2_k, const void *w1_v, const void *w2_v,
                           int32_t hidden, int32_t activation, const void *q, void *out,
                           float *lse_out, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/* Closed-form fit of a linear predictor to the stage-1 reconstruction loss
 * (Sec. "Training Details": || C_hat_drop - C_drop ||^2).  For a linear map the
 * minimiser is the least-squares solution
 *   W = argmin || [C_global ; C_local] W - C_drop ||_F^2 + ridge ||W||_F^2
 * over n_rows token rows.  The Gram matrices X^T X and X^T C_drop are formed on
 * MFMA (bf16 inputs, fp32 accumulation) and the normal equations are solved by
 * conjugate gradients in fp32 on the GPU (one step length for all columns).
 *   anchor_rows : device [n_rows, D] bf16, the anchor layer's rows (K or V)
 *   target_rows : device [n_rows, D] bf16, the target layer's FULL rows of the same
 *                 tokens (first m dims = C_local, the rest = C_drop)
 *   n_rows      : multiple of 64
 *   w_out       : device [D + m, D - m] bf16
 *   max_iters, tol : stop after max_iters steps or once ||residual||_F <= tol ||X^T C_drop||_F
 *   iters_out, rel_residual_out : HOST, optional
 * A training-side utility: synchronous (it reads two scalars back per step).
 * bf16 only; workspace from echokv_fit_workspace_bytes. */
size_t echokv_fit_workspace_bytes(const echokv_shape *shape, int64_t n_rows);
int echokv_fit_linear(const echokv_shape *shape, const void *anchor_rows,
                      const void *target_rows, int64_t n_rows, float ridge,
                      int32_t max_iters, float tol, void *w_out, void *workspace,
                      size_t workspace_bytes, int32_t *iters_out,
                      float *rel_residual_out, void *hip_stream);

/* Causal chunk of T_q queries of sequence `seq` (Eq. 7 with a causal mask):
 * query i sits at position q_pos0 + i and attends cached tokens
 * 0 .. q_pos0 + i inclusive, all read from the compressed cache (predicted
 * where dropped).  Requires seq_len[seq] >= q_pos0 + T_q: the chunk's own K/V
 * have been appended already.
 *   q   : device [T_q, H_q, d];  out : device [T_q, H_q, d];
 *   lse_out : device [T_q, H_q] fp32 or NULL. */
int echokv_prefill_attn(const echokv_shape *shape, const echokv_layer_cache *anchor,
                        const echokv_layer_cache *target, const void *w_k,
                        const void *w_v, int32_t seq, const void *q, int32_t T_q,
                        int32_t q_pos0, void *out, float *lse_out, void *workspace,
                        size_t workspace_bytes, void *hip_stream);

/* echokv_prefill_attn with the rotary embedding of the paper's inference (Sec.
 * "Network Architecture": the caches hold pre-rotation keys): with
 * extras->rope_cos / rope_sin set, the key of cached token j -- retained or
 * predicted -- is rotated to position j before the dot products, with the
 * pairing and table layout described above echokv_decode_extras; q must come in
 * already rotated (query i to position q_pos0 + i); rope_positions >=
 * q_pos0 + T_q.  A prefill chunk reads the compressed cache only: extras with
 * window pointers are refused (ECHOKV_ERR_UNSUPPORTED).  extras == NULL or no
 * tables: the same as echokv_prefill_attn.  Same workspace size.  (bf16: the
 * rotated keys are rounded to bf16 once more before the attention products.) */
int echokv_prefill_attn_ex(const echokv_shape *shape, const echokv_layer_cache *anchor,
                           const echokv_layer_cache *target, const void *w_k,
                           const void *w_v, int32_t seq, const void *q, int32_t T_q,
                           int32_t q_pos0, const echokv_decode_extras *extras, void *out,
                           float *lse_out, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/* Measurement aid (no paper passage: it exists so that a benchmark can report
 * the duration of the kernel that dominates echokv_decode_attn, the fused
 * predictor-product + attention kernel, separately from the whole call).
 * While enabled, every echokv_decode_attn call records a HIP event pair on its
 * stream around that kernel's launch.  echokv_profile_read waits for the
 * recorded events, adds up the elapsed times, returns them with the number of
 * launches, and forgets them.  Not thread safe; keep it off in production. */
int echokv_profile_enable(int on);
int echokv_profile_read(double *total_ms, int64_t *launches);
/* The same for a prefill chunk: channel 1 = the chunk's predictor product (Eq. 3
 * for every visible token), channel 2 = its causal attention kernel (Eq. 7);
 * channel 0 is what echokv_profile_read returns.  The recorder is one
 * process-wide list: do not call the library from two threads while it is on. */
int echokv_profile_read_channel(int channel, double *total_ms, int64_t *launches);

/* Measurement aid: the rate at which a plain kernel streams `bytes` of device
 * memory at `buf` (16-byte aligned, at least 403 MB to mean anything; the
 * tail beyond a multiple of 384 MiB is not read) through the chip, best of
 * `repeats` timed passes on the default stream, in GB/s.  The yardstick for the
 * HBM-bound kernels: what the memory system delivers to the simplest possible
 * reader, as opposed to the nominal peak.  Synchronous. */
int echokv_profile_stream_read(const void *buf, size_t bytes, int32_t repeats,
                               double *gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* ECHOKV_H */
