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
  * keys are position-free on this path (no rotary embedding is applied);
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
