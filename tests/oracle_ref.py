"""Bridges seeded Inputs (torch CPU tensors in the storage dtype) to the fp64
NumPy oracle.  Upcasting the stored values is the only conversion."""
import numpy as np

from oracle import echokv_oracle as orc


def f64(t):
    return t.double().numpy()


def seq_arrays(inp, b):
    r = inp.rows(b)
    return f64(inp.K_a[r]), f64(inp.V_a[r]), f64(inp.K_r[r]), f64(inp.V_r[r])


def weights(inp):
    if inp.w.d_out == 0:
        return None, None
    return f64(inp.W_K), f64(inp.W_V)


def decode_ref(inp, seqs=None, scale=None):
    """(out [n, H_q, d], lse [n, H_q]) for the chosen decode sequences."""
    seqs = range(inp.n_decode) if seqs is None else seqs
    W_K, W_V = weights(inp)
    outs, lses = [], []
    for b in seqs:
        K_a, V_a, K_r, V_r = seq_arrays(inp, b)
        o, l = orc.echokv_decode(f64(inp.q[b]), K_a, V_a, K_r, V_r, W_K, W_V,
                                 inp.w.n_kv_heads, scale)
        outs.append(o); lses.append(l)
    return np.stack(outs), np.stack(lses)


def prefill_ref(inp, scale=None):
    b = inp.n_decode
    K_a, V_a, K_r, V_r = seq_arrays(inp, b)
    W_K, W_V = weights(inp)
    return orc.echokv_prefill(f64(inp.q_prefill), K_a, V_a, K_r, V_r, W_K, W_V,
                              inp.w.n_kv_heads, inp.q_pos0, scale)


def prefill_paper_ref(inp, rope, scale=None):
    """rope = (cos, sin) torch fp32 tables."""
    b = inp.n_decode
    K_a, V_a, K_r, V_r = seq_arrays(inp, b)
    W_K, W_V = weights(inp)
    return orc.echokv_prefill_paper(f64(inp.q_prefill), K_a, V_a, K_r, V_r, W_K, W_V,
                                    inp.w.n_kv_heads, inp.q_pos0, scale,
                                    rope=(f64(rope[0]), f64(rope[1])))


def reconstruct_ref(inp, b, t0, t1):
    K_a, V_a, K_r, V_r = seq_arrays(inp, b)
    W_K, W_V = weights(inp)
    return (orc.reconstruct(K_a[t0:t1], K_r[t0:t1], W_K),
            orc.reconstruct(V_a[t0:t1], V_r[t0:t1], W_V))


def decode_head_ref(inp, b, h, scale=None):
    K_a, V_a, K_r, V_r = seq_arrays(inp, b)
    W_K, W_V = weights(inp)
    w = inp.w
    return orc.echokv_decode_head(f64(inp.q[b, h]), K_a, V_a, K_r, V_r, W_K, W_V,
                                  h // w.group, w.head_dim, scale)


def decode_paper_ref(inp, rope=None, window=None, seqs=None, scale=None):
    """Paper-faithful decode: rope = (cos, sin) torch fp32 tables; window =
    (win_k, win_v, n_sink, n_recent) with torch [n_decode, rows, D] buffers."""
    seqs = range(inp.n_decode) if seqs is None else seqs
    W_K, W_V = weights(inp)
    r = None if rope is None else (f64(rope[0]), f64(rope[1]))
    outs, lses = [], []
    for b in seqs:
        K_a, V_a, K_r, V_r = seq_arrays(inp, b)
        wnd = None if window is None else (f64(window[0][b]), f64(window[1][b]), window[2], window[3])
        o, l = orc.echokv_decode_paper(f64(inp.q[b]), K_a, V_a, K_r, V_r, W_K, W_V,
                                       inp.w.n_kv_heads, scale, rope=r, window=wnd)
        outs.append(o); lses.append(l)
    return np.stack(outs), np.stack(lses)


def decode_mlp_ref(inp, weights, act, seqs=None, scale=None):
    """weights = (W1_K, W2_K, W1_V, W2_V) torch tensors; act = "relu" | "silu"."""
    seqs = range(inp.n_decode) if seqs is None else seqs
    W = [f64(t) for t in weights]
    outs, lses = [], []
    for b in seqs:
        K_a, V_a, K_r, V_r = seq_arrays(inp, b)
        o, l = orc.echokv_decode_mlp(f64(inp.q[b]), K_a, V_a, K_r, V_r, W[0], W[1], W[2], W[3],
                                     inp.w.n_kv_heads, act, scale)
        outs.append(o); lses.append(l)
    return np.stack(outs), np.stack(lses)
