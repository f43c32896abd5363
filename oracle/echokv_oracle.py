"""CPU oracle for EchoKV attention over a compressed KV cache (fp64, NumPy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
library is checked against.  It shares no code with the library, imports
nothing from it, and must never be called from the product path: only the
tests, the smoke check and the benchmark's cpu_baseline leg may use it.

What is defined here, following the paper's notation
(Sec. "Network Architecture", Eq. 1-4; Sec. "Training Details", Eq. 6-7;
Appendix "Analysis of QK-KL Divergence Loss" for softmax(QK^T/sqrt(d))):

  C_global = full flattened cache of the group's first (anchor) layer   Eq. 1
  C_local  = C[:, :m], first m flattened dims of the target layer       Eq. 2
  C_hat    = [C_global ; C_local] W                                     Eq. 3
  C_drop   = C[:, m:] (never stored; what C_hat stands in for)          Eq. 4
  X_tilde  = Reshape([X_local ; X_hat_drop]),  X in {K, V}              Eq. 6
  out      = A(Q, K_tilde, V_tilde) = softmax(Q K_tilde^T / sqrt(d)) V_tilde   Eq. 7

Readings taken where the paper is silent (each also listed in the design notes):
  * the predictor is a bias-free linear map, applied per token in row form
    y = x W with W of shape [d_in, d_out]; keys and values have separate W;
  * flattening is head-major: flattened index g*d + i is feature i of KV head g;
  * query head h reads KV head h // G, G = H_q / H_kv;
  * keys are position-free on the base path (no rotary embedding is applied);
    echokv_decode_paper adds what the paper's own inference does on top: the
    cache holds keys from before the rotary embedding (Sec. "Network
    Architecture"), so the embedding is applied to the rebuilt keys, by token
    position, just before Eq. 7; and the first 4 / latest 128 tokens of the
    target layer are kept uncompressed (Sec. "Experimental Setting", paragraph
    "Implement details").  The
    pairing of rotated features (i with i + d/2) and the ring placement of the
    latest tokens are this build's readings: the paper fixes neither;
  * the one-hidden-layer predictor of Appendix "Prediction Network Architecture"
    is read as C_hat = act([C_global ; C_local] W1) W2, bias-free like the
    linear one, act = ReLU or SiLU (the paper names no activation);
  * a prefill query at chunk offset i attends cached tokens 0 .. q_pos0 + i,
    all of them taken from the compressed cache (reconstructed where dropped).

Two codings: the vectorised one (BLAS matmul per step) and a scalar brute force
for tiny shapes.  All arithmetic is float64; inputs are the stored values
upcast, with no further rounding anywhere.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------
# shape / layout arithmetic (Appendix "Compression-Ratio Configurations")
# --------------------------------------------------------------------------
def predictor_dims(D: int, m: int) -> Tuple[int, int]:
    """(d_in, d_out): the predictor sees D anchor dims plus m local dims and
    emits the D - m dropped dims (Eq. 3, Eq. 4)."""
    if not 0 <= m <= D:
        raise ValueError("need 0 <= m <= D")
    return D + m, D - m


def compression_ratio(D: int, m: int, S: int) -> float:
    """Stored dims over full dims for one group of S layers: the anchor keeps
    D, each of the S-1 targets keeps m."""
    return (D + m * (S - 1)) / (D * S)


def predictor_param_count(n_layers: int, S: int, D: int, m: int,
                          bias: bool = False) -> int:
    """Parameters of all predictors of a model: one W for K and one for V in
    every non-anchor layer."""
    d_in, d_out = predictor_dims(D, m)
    n_target = n_layers - n_layers // S
    per = d_in * d_out + (d_out if bias else 0)
    return n_target * 2 * per


# --------------------------------------------------------------------------
# cache layout (Eq. 1, Eq. 2; dropping at write time, Sec. "Throughput Analysis")
# --------------------------------------------------------------------------
def cache_append(cache: np.ndarray, seq_start: int, seq_len: int,
                 new_rows: np.ndarray) -> int:
    """Append full-width rows to one sequence of a layer cache of width
    cache.shape[1]: only the first `width` flattened dims are kept (width = D
    for an anchor layer, m for a target layer).  Returns the new length."""
    width = cache.shape[1]
    n = new_rows.shape[0]
    cache[seq_start + seq_len: seq_start + seq_len + n, :] = new_rows[:, :width]
    return seq_len + n


def cache_compress(full_cache: np.ndarray, m: int) -> np.ndarray:
    """Full -> compressed switch of a target layer (Sec. "Overview of EchoKV"):
    the dims [m, D) are evicted, the first m flattened dims stay (Eq. 2)."""
    return np.array(full_cache[:, :m], copy=True)


# --------------------------------------------------------------------------
# reconstruction (Eq. 3, Eq. 6)
# --------------------------------------------------------------------------
def predictor_input(C_anchor: np.ndarray, C_local: np.ndarray) -> np.ndarray:
    """Per-token predictor input rows [C_global ; C_local], anchor dims first."""
    return np.concatenate([np.asarray(C_anchor, F64), np.asarray(C_local, F64)],
                          axis=1)


def reconstruct(C_anchor: np.ndarray, C_local: np.ndarray,
                W: Optional[np.ndarray]) -> np.ndarray:
    """C_tilde [L, D] = [C_local ; [C_anchor ; C_local] W], retained dims first.
    With m == D there is nothing to predict and W is unused."""
    C_local = np.asarray(C_local, F64)
    D = C_anchor.shape[1]
    m = C_local.shape[1]
    if m == D:
        return C_local.copy()
    X = predictor_input(C_anchor, C_local)
    W = np.asarray(W, F64)
    if W.shape != (D + m, D - m):
        raise ValueError(f"W must be [{D + m}, {D - m}], got {W.shape}")
    C_hat = X @ W
    return np.concatenate([C_local, C_hat], axis=1)


# --------------------------------------------------------------------------
# attention (Eq. 7)
# --------------------------------------------------------------------------
def _scale(d: int, scale: Optional[float]) -> float:
    return 1.0 / math.sqrt(d) if scale is None or scale <= 0 else float(scale)


def attention_rows(Q: np.ndarray, K: np.ndarray, V: np.ndarray, n_kv_heads: int,
                   scale: Optional[float] = None,
                   visible: Optional[Sequence[int]] = None):
    """softmax(q K_g^T * scale) V_g for every query row and head.

    Q [T, H_q, d]; K, V [L, D] flattened head-major.  visible[t] = number of
    leading tokens query t may attend (default: all L).  Returns
    (out [T, H_q, d], lse [T, H_q], P [T, H_q, L]) with P the softmax rows.
    """
    Q = np.asarray(Q, F64)
    T, H_q, d = Q.shape
    L = K.shape[0]
    G = H_q // n_kv_heads
    sc = _scale(d, scale)
    Kh = np.asarray(K, F64).reshape(L, n_kv_heads, d)
    Vh = np.asarray(V, F64).reshape(L, n_kv_heads, d)
    out = np.zeros((T, H_q, d), F64)
    lse = np.zeros((T, H_q), F64)
    P = np.zeros((T, H_q, L), F64)
    for h in range(H_q):
        g = h // G
        s = (Q[:, h, :] @ Kh[:, g, :].T) * sc                 # [T, L]
        if visible is not None:
            for t in range(T):
                s[t, int(visible[t]):] = -np.inf
        mx = s.max(axis=1, keepdims=True)
        e = np.exp(s - mx)
        z = e.sum(axis=1, keepdims=True)
        p = e / z
        P[:, h, :] = p
        out[:, h, :] = p @ Vh[:, g, :]
        lse[:, h] = (mx + np.log(z))[:, 0]
    return out, lse, P


def echokv_decode(q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int,
                  scale: Optional[float] = None):
    """One decode query per head over one sequence's compressed cache.
    q [H_q, d]; K_a, V_a [L, D]; K_r, V_r [L, m].  Returns (out [H_q, d], lse [H_q])."""
    K_t = reconstruct(K_a, K_r, W_K)
    V_t = reconstruct(V_a, V_r, W_V)
    o, lse, _ = attention_rows(np.asarray(q, F64)[None], K_t, V_t, n_kv_heads, scale)
    return o[0], lse[0]


def echokv_decode_head(q_h, K_a, V_a, K_r, V_r, W_K, W_V, g: int, d: int,
                       scale: Optional[float] = None):
    """One query head against KV head g only (for spot checks at sizes where the
    whole layer is too slow): the head's d columns of K_tilde / V_tilde are the
    stored ones if g*d < m, else columns [g*d - m, g*d - m + d) of the predictor
    output (Eq. 3, Eq. 6); then Eq. 7 for that head.  Returns (out [d], lse)."""
    m = K_r.shape[1]
    lo = g * d
    if lo < m:
        K_g = np.asarray(K_r, F64)[:, lo:lo + d]
        V_g = np.asarray(V_r, F64)[:, lo:lo + d]
    else:
        cols = slice(lo - m, lo - m + d)
        K_g = predictor_input(K_a, K_r) @ np.asarray(W_K, F64)[:, cols]
        V_g = predictor_input(V_a, V_r) @ np.asarray(W_V, F64)[:, cols]
    o, lse, _ = attention_rows(np.asarray(q_h, F64)[None, None, :], K_g, V_g, 1, scale)
    return o[0, 0], lse[0, 0]


def echokv_prefill(Q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int, q_pos0: int,
                   scale: Optional[float] = None):
    """Causal chunk: query i sits at position q_pos0 + i and attends cached
    tokens 0 .. q_pos0 + i inclusive; the cache already holds the chunk's own
    tokens.  Q [T_q, H_q, d].  Returns (out [T_q, H_q, d], lse [T_q, H_q])."""
    T_q = Q.shape[0]
    L = K_a.shape[0]
    if q_pos0 < 0 or q_pos0 + T_q > L:
        raise ValueError("cache must already hold the chunk: need q_pos0 + T_q <= L")
    K_t = reconstruct(K_a, K_r, W_K)
    V_t = reconstruct(V_a, V_r, W_V)
    vis = [q_pos0 + i + 1 for i in range(T_q)]
    o, lse, _ = attention_rows(Q, K_t, V_t, n_kv_heads, scale, visible=vis)
    return o, lse


# --------------------------------------------------------------------------
# split-K merge: exact re-association of the softmax-weighted sum over a
# partition of the tokens (not in the paper; used by flash-decoding designs)
# --------------------------------------------------------------------------
def merge_partials(m_s: np.ndarray, l_s: np.ndarray, o_s: np.ndarray):
    """Partials over n splits: m_s [n] running max, l_s [n] sum of exp(s - m_s),
    o_s [n, d] sum of exp(s - m_s) v.  Returns (out [d], lse)."""
    m_s = np.asarray(m_s, F64); l_s = np.asarray(l_s, F64); o_s = np.asarray(o_s, F64)
    M = m_s.max()
    wgt = np.exp(m_s - M)
    denom = (wgt * l_s).sum()
    return (wgt[:, None] * o_s).sum(axis=0) / denom, M + math.log(denom)


# --------------------------------------------------------------------------
# brute force, scalar loops only (tiny shapes)
# --------------------------------------------------------------------------
def brute_force_prefill(Q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int,
                        q_pos0: int, scale: Optional[float] = None):
    """Same function as echokv_prefill, written as nested scalar loops straight
    from Eq. 3, 6, 7.  With T_q = 1 and q_pos0 = L - 1 it is the decode case."""
    Q = np.asarray(Q, F64)
    T_q, H_q, d = Q.shape
    L, D = K_a.shape
    m = K_r.shape[1]
    G = H_q // n_kv_heads
    sc = _scale(d, scale)

    def rebuilt(C_a, C_r, W, j, col):            # flattened dim `col` of token j
        if col < m:
            return float(C_r[j][col])
        acc = 0.0
        for k in range(D + m):                    # [anchor ; local] order
            x = float(C_a[j][k]) if k < D else float(C_r[j][k - D])
            acc += x * float(W[k][col - m])
        return acc

    out = [[[0.0] * d for _ in range(H_q)] for _ in range(T_q)]
    lse = [[0.0] * H_q for _ in range(T_q)]
    for t in range(T_q):
        n_vis = q_pos0 + t + 1
        for h in range(H_q):
            g = h // G
            s = []
            for j in range(n_vis):
                dot = 0.0
                for i in range(d):
                    dot += float(Q[t][h][i]) * rebuilt(K_a, K_r, W_K, j, g * d + i)
                s.append(dot * sc)
            mx = max(s)
            e = [math.exp(x - mx) for x in s]
            z = sum(e)
            for i in range(d):
                acc = 0.0
                for j in range(n_vis):
                    acc += (e[j] / z) * rebuilt(V_a, V_r, W_V, j, g * d + i)
                out[t][h][i] = acc
            lse[t][h] = mx + math.log(z)
    return np.array(out, F64), np.array(lse, F64)


def brute_force_decode(q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int,
                       scale: Optional[float] = None):
    L = K_a.shape[0]
    o, lse = brute_force_prefill(np.asarray(q, F64)[None], K_a, V_a, K_r, V_r,
                                 W_K, W_V, n_kv_heads, L - 1, scale)
    return o[0], lse[0]


# --------------------------------------------------------------------------
# paper-faithful decode: rotary embedding after reconstruction, and a window
# of uncompressed tokens (Sec. "Network Architecture": predictor inputs are
# the keys BEFORE the rotary embedding; Sec. "Experimental Setting", paragraph
# "Implement details": the first 4 tokens and the most recent 128 tokens of a
# sequence are exempt from compression)
# --------------------------------------------------------------------------
def rope_rotate(X: np.ndarray, positions: Sequence[int], cos: np.ndarray, sin: np.ndarray,
                n_heads: int) -> np.ndarray:
    """Rotary embedding of flattened head-major rows X [L, n_heads * d].

    Row j is rotated by the angles of table row positions[j]; cos, sin are
    [P, d/2] (the caller's tables: angle of feature pair i at position p).
    Feature i of a head is paired with feature i + d/2:
        x'_i       = x_i cos_i - x_{i+d/2} sin_i
        x'_{i+d/2} = x_{i+d/2} cos_i + x_i sin_i
    """
    X = np.asarray(X, F64)
    L = X.shape[0]
    d = X.shape[1] // n_heads
    h = d // 2
    pos = np.asarray(positions, np.int64)
    c = np.asarray(cos, F64)[pos][:, None, :]          # [L, 1, d/2]
    s = np.asarray(sin, F64)[pos][:, None, :]
    Xh = X.reshape(L, n_heads, d)
    a, b = Xh[:, :, :h], Xh[:, :, h:]
    out = np.empty_like(Xh)
    out[:, :, :h] = a * c - b * s
    out[:, :, h:] = b * c + a * s
    return out.reshape(L, n_heads * d)


def window_row(p: int, n_sink: int, n_recent: int) -> int:
    """Row of the uncompressed window that holds position p: the first n_sink
    positions have a row each, later positions share a ring of n_recent rows."""
    return p if p < n_sink else n_sink + (p - n_sink) % n_recent


def in_window(p: int, L: int, n_sink: int, n_recent: int) -> bool:
    """Is position p of a length-L sequence kept uncompressed?"""
    return p < n_sink or p >= L - n_recent


def window_append(win: np.ndarray, L_before: int, rows: np.ndarray, n_sink: int, n_recent: int):
    """Write full-width rows of new tokens (positions L_before, L_before+1, ...)
    into the window [n_sink + n_recent, D], in place; the ring overwrites the
    token that leaves the local window."""
    for i in range(rows.shape[0]):
        p = L_before + i
        if p < n_sink or n_recent > 0:
            win[window_row(p, n_sink, n_recent)] = rows[i]


def rebuilt_with_window(C_a, C_r, W, win, n_sink: int, n_recent: int) -> np.ndarray:
    """C_tilde [L, D]: reconstruction (Eq. 3, 6) everywhere except the window
    positions, which take their stored uncompressed rows."""
    C_t = reconstruct(C_a, C_r, W)
    L = C_t.shape[0]
    if win is not None:
        win = np.asarray(win, F64)
        for p in range(L):
            if in_window(p, L, n_sink, n_recent):
                C_t[p] = win[window_row(p, n_sink, n_recent)]
    return C_t


def echokv_decode_paper(q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int,
                        scale: Optional[float] = None,
                        rope: Optional[Tuple[np.ndarray, np.ndarray]] = None,
                        window: Optional[Tuple[np.ndarray, np.ndarray, int, int]] = None):
    """Decode over one sequence as the paper's inference runs it.

    rope = (cos, sin) tables [P, d/2]: cached keys are pre-rotation; token j's
    rebuilt key is rotated to position j before the dot product.  q must come
    in already rotated to its own position.  window = (win_k, win_v, n_sink,
    n_recent): full-width pre-rotation rows of the target layer for the first
    n_sink and the latest n_recent positions, laid out by window_row().
    Returns (out [H_q, d], lse [H_q])."""
    wk = wv = None
    n_sink = n_recent = 0
    if window is not None:
        wk, wv, n_sink, n_recent = window
    K_t = rebuilt_with_window(K_a, K_r, W_K, wk, n_sink, n_recent)
    V_t = rebuilt_with_window(V_a, V_r, W_V, wv, n_sink, n_recent)
    if rope is not None:
        K_t = rope_rotate(K_t, range(K_t.shape[0]), rope[0], rope[1], n_kv_heads)
    o, lse, _ = attention_rows(np.asarray(q, F64)[None], K_t, V_t, n_kv_heads, scale)
    return o[0], lse[0]


def echokv_prefill_paper(Q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int, q_pos0: int,
                         scale: Optional[float] = None,
                         rope: Optional[Tuple[np.ndarray, np.ndarray]] = None):
    """echokv_prefill with the rotary embedding of the paper's inference: cached
    keys are pre-rotation, token j's rebuilt key is rotated to position j before
    the dot products; Q [T_q, H_q, d] must come in already rotated (query i to
    position q_pos0 + i).  Returns (out [T_q, H_q, d], lse [T_q, H_q])."""
    T_q = Q.shape[0]
    L = K_a.shape[0]
    if q_pos0 < 0 or q_pos0 + T_q > L:
        raise ValueError("cache must already hold the chunk: need q_pos0 + T_q <= L")
    K_t = reconstruct(K_a, K_r, W_K)
    V_t = reconstruct(V_a, V_r, W_V)
    if rope is not None:
        K_t = rope_rotate(K_t, range(L), rope[0], rope[1], n_kv_heads)
    vis = [q_pos0 + i + 1 for i in range(T_q)]
    o, lse, _ = attention_rows(Q, K_t, V_t, n_kv_heads, scale, visible=vis)
    return o, lse


def brute_force_decode_paper(q, K_a, V_a, K_r, V_r, W_K, W_V, n_kv_heads: int,
                             scale=None, rope=None, window=None):
    """echokv_decode_paper again as scalar loops (tiny shapes)."""
    q = np.asarray(q, F64)
    H_q, d = q.shape
    L, D = K_a.shape
    m = K_r.shape[1]
    G = H_q // n_kv_heads
    sc = _scale(d, scale)
    half = d // 2
    n_sink = n_recent = 0
    if window is not None:
        win_k, win_v, n_sink, n_recent = window

    def stored(C_a, C_r, W, win, j, col):
        if window is not None and (j < n_sink or j >= L - n_recent):
            r = j if j < n_sink else n_sink + (j - n_sink) % n_recent
            return float(win[r][col])
        if col < m:
            return float(C_r[j][col])
        acc = 0.0
        for k in range(D + m):
            x = float(C_a[j][k]) if k < D else float(C_r[j][k - D])
            acc += x * float(W[k][col - m])
        return acc

    def key(j, g, i):
        x = stored(K_a, K_r, W_K, win_k if window is not None else None, j, g * d + i)
        if rope is None:
            return x
        if i < half:
            y = stored(K_a, K_r, W_K, win_k if window is not None else None, j, g * d + i + half)
            return x * float(rope[0][j][i]) - y * float(rope[1][j][i])
        y = stored(K_a, K_r, W_K, win_k if window is not None else None, j, g * d + i - half)
        return x * float(rope[0][j][i - half]) + y * float(rope[1][j][i - half])

    out = [[0.0] * d for _ in range(H_q)]
    lse = [0.0] * H_q
    for h in range(H_q):
        g = h // G
        s = []
        for j in range(L):
            dot = 0.0
            for i in range(d):
                dot += float(q[h][i]) * key(j, g, i)
            s.append(dot * sc)
        mx = max(s)
        e = [math.exp(x - mx) for x in s]
        z = sum(e)
        for i in range(d):
            acc = 0.0
            for j in range(L):
                acc += (e[j] / z) * stored(V_a, V_r, W_V, win_v if window is not None else None, j, g * d + i)
            out[h][i] = acc
        lse[h] = mx + math.log(z)
    return np.array(out, F64), np.array(lse, F64)


# --------------------------------------------------------------------------
# one-hidden-layer predictor (Appendix "Prediction Network Architecture":
# a parameter-matched hidden width, or hidden width = predictor input width)
# --------------------------------------------------------------------------
def activation(x: np.ndarray, kind: str) -> np.ndarray:
    x = np.asarray(x, F64)
    if kind == "relu":
        return np.maximum(x, 0.0)
    if kind == "silu":
        return x / (1.0 + np.exp(-x))
    raise ValueError(f"unknown activation {kind!r}")


def reconstruct_mlp(C_anchor, C_local, W1, W2, act: str = "relu") -> np.ndarray:
    """C_tilde [L, D] = [C_local ; act([C_anchor ; C_local] W1) W2], retained dims
    first (Eq. 3 with the linear map replaced by the two-layer one, Eq. 6).
    W1 [D + m, hidden], W2 [hidden, D - m]."""
    C_local = np.asarray(C_local, F64)
    D = C_anchor.shape[1]
    m = C_local.shape[1]
    W1 = np.asarray(W1, F64); W2 = np.asarray(W2, F64)
    if W1.shape[0] != D + m or W2.shape != (W1.shape[1], D - m):
        raise ValueError("need W1 [D + m, hidden] and W2 [hidden, D - m]")
    H = activation(predictor_input(C_anchor, C_local) @ W1, act)
    return np.concatenate([C_local, H @ W2], axis=1)


def echokv_decode_mlp(q, K_a, V_a, K_r, V_r, W1_K, W2_K, W1_V, W2_V, n_kv_heads: int,
                      act: str = "relu", scale: Optional[float] = None):
    """Decode over one sequence with the one-hidden-layer predictor.
    Returns (out [H_q, d], lse [H_q])."""
    K_t = reconstruct_mlp(K_a, K_r, W1_K, W2_K, act)
    V_t = reconstruct_mlp(V_a, V_r, W1_V, W2_V, act)
    o, lse, _ = attention_rows(np.asarray(q, F64)[None], K_t, V_t, n_kv_heads, scale)
    return o[0], lse[0]


def mlp_param_matched_hidden(D: int, m: int, multiple: int = 64) -> int:
    """Hidden width that keeps the two-layer predictor's parameter count closest to
    the linear one's: hidden * (d_in + d_out) ~ d_in * d_out, rounded to `multiple`."""
    d_in, d_out = predictor_dims(D, m)
    h = d_in * d_out / (d_in + d_out)
    return max(multiple, int(round(h / multiple)) * multiple)


# --------------------------------------------------------------------------
# stage-1 fit of the linear predictor (Sec. "Training Details", the
# reconstruction loss || C_hat_drop - C_drop ||^2): for a linear map the
# minimiser has a closed form, the least-squares solution
# --------------------------------------------------------------------------
def fit_linear(C_anchor: np.ndarray, C_target_full: np.ndarray, m: int, ridge: float = 0.0) -> np.ndarray:
    """W [D + m, D - m] = argmin || [C_anchor ; C_target[:, :m]] W - C_target[:, m:] ||_F^2
    + ridge ||W||_F^2 over the given token rows."""
    C_a = np.asarray(C_anchor, F64); C_t = np.asarray(C_target_full, F64)
    X = predictor_input(C_a, C_t[:, :m])
    Y = C_t[:, m:]
    if ridge == 0.0:
        return np.linalg.lstsq(X, Y, rcond=None)[0]
    return np.linalg.solve(X.T @ X + ridge * np.eye(X.shape[1]), X.T @ Y)


def reconstruction_loss(C_anchor, C_target_full, m: int, W) -> float:
    """Mean squared error of the rebuilt dims (the stage-1 loss per element)."""
    C_t = np.asarray(C_target_full, F64)
    C_hat = predictor_input(C_anchor, C_t[:, :m]) @ np.asarray(W, F64)
    return float(np.mean((C_hat - C_t[:, m:]) ** 2))
