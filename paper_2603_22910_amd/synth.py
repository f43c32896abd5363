"""Seeded synthetic workloads for the EchoKV decode hot path.

This module only draws random inputs and lays them out the way the compressed
cache stores them.  It contains none of the method's arithmetic (no predictor
product, no softmax, no attention): both the CPU oracle's tests and the HIP
path's tests/bench take their inputs from here, and that is all they share.

Workload shapes follow the paper's models (per-layer flattened KV width
D = H_kv * d, Appendix "Compression-Ratio Configurations") and its long-context
evaluation lengths (Sec. "Experimental Setting": 32K RULER, model-max
LongBench; Sec. "Throughput Analysis": batch 8 up to 36K tokens).  The five
named configurations are the benchmark's; values are synthetic.

Recipe (all draws fp32 on the CPU, then rounded ONCE to the storage dtype):
  lengths  : own generator seeded (seed, "len"); fixed list, or log-uniform
             L_b = floor(lo * (hi/lo)**u_b), u_b ~ U[0,1)
  pool     : sequence b occupies rows [seq_start[b], seq_start[b]+L_b) of one
             token-major pool; seq_start = prefix sums of L_b rounded up to
             ROW_ALIGN rows.  Gap rows are zero.
  anchor   : K_a, V_a ~ N(0,1), [pool, D]
  retained : T[:, :m] = A @ M1 + 0.1 * E1, M1 ~ N(0, std 1/sqrt(D)) [D, m],
             E1 ~ N(0,1), separately for K and V (the target layer's kept
             prefix is correlated with the anchor layer, as the method assumes)
  weights  : W_K, W_V ~ N(0, std 1/sqrt(d_in)), [d_in, d_out] row-major
  queries  : q ~ N(0,1), [B, H_q, d]; prefill chunk q_p ~ N(0,1), [T_q, H_q, d]
Every tensor has its own generator seeded by (seed, tag); the row-indexed ones
(K_a, V_a, E1) are drawn in fixed chunks of _CHUNK_ROWS rows, each chunk from
its own generator seeded by (seed, tag, chunk index), so a tensor does not
change when another one's shape does and chunks can be drawn in parallel.
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
import hashlib
import math
import os
from typing import Dict, List, Optional, Sequence

import torch

ROW_ALIGN = 256          # pool rows reserved per sequence are a multiple of this
_CHUNK_ROWS = 2048       # rows per generator chunk (part of the recipe)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                    # "bf16" | "f32"
    n_q_heads: int                # H_q
    n_kv_heads: int               # H_kv
    head_dim: int                 # d
    n_retained: int               # m  (flattened dims the target layer keeps)
    seed: int
    seq_lens: Optional[Sequence[int]] = None     # fixed lengths, or
    batch: int = 0                                # log-uniform lengths
    len_lo: int = 0
    len_hi: int = 0
    prefill_len: int = 0          # >0: one extra sequence of this many tokens
    prefill_q: int = 0            # queries in the prefill chunk (last rows)

    @property
    def D(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def d_in(self) -> int:
        return self.D + self.n_retained

    @property
    def d_out(self) -> int:
        return self.D - self.n_retained

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"bf16": torch.bfloat16, "f32": torch.float32}[self.dtype]

    @property
    def elem_size(self) -> int:
        return {"bf16": 2, "f32": 4}[self.dtype]

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (reduced-size test cases)."""
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (index == seed).
CONFIGS: Dict[int, Workload] = {
    0: Workload("cfg0_tiny_f32", "f32", 8, 8, 64, 256, seed=0, seq_lens=(512,)),
    1: Workload("cfg1_7b_mha_r50_b8_l4096", "bf16", 32, 32, 128, 2048, seed=1,
                seq_lens=(4096,) * 8),
    2: Workload("cfg2_7b_mha_r25_b4_l32768", "bf16", 32, 32, 128, 1024, seed=2,
                seq_lens=(32768,) * 4),
    3: Workload("cfg3_8b_gqa_r50_b1_l131072", "bf16", 32, 8, 128, 512, seed=3,
                seq_lens=(131072,)),
    4: Workload("cfg4_7b_mha_r50_ragged_b32", "bf16", 32, 32, 128, 2048, seed=4,
                batch=32, len_lo=1024, len_hi=65536,
                prefill_len=8192, prefill_q=8192),
}


def _gen(seed: int, tag: str) -> torch.Generator:
    h = hashlib.sha256(f"echokv-synth/{seed}/{tag}".encode()).digest()
    g = torch.Generator(device="cpu")
    g.manual_seed(int.from_bytes(h[:8], "little") & ((1 << 63) - 1))
    return g


def draw_lengths(w: Workload) -> List[int]:
    """Decode-batch context lengths L_b (the prefill sequence is not included)."""
    if w.seq_lens is not None:
        return [int(x) for x in w.seq_lens]
    u = torch.rand(w.batch, generator=_gen(w.seed, "len"), dtype=torch.float64)
    ratio = w.len_hi / w.len_lo
    return [min(w.len_hi, int(math.floor(w.len_lo * ratio ** float(x)))) for x in u]


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


_DRAW_THREADS = 8        # chunks drawn concurrently (does not affect the values)


def _draw_rows(r0: int, r1: int, cols: int, seed: int, tag: str) -> torch.Tensor:
    """Rows [r0, r1) of a [*, cols] N(0,1) tensor whose chunk c (rows
    c*_CHUNK_ROWS ...) comes from its own generator (seed, tag, c).  r0 must be
    chunk-aligned.  Chunks are drawn on a few threads."""
    out = torch.empty(r1 - r0, cols, dtype=torch.float32)
    jobs = [(c0 // _CHUNK_ROWS, c0, min(r1, c0 + _CHUNK_ROWS)) for c0 in range(r0, r1, _CHUNK_ROWS)]

    def job(j):
        i, c0, c1 = j
        torch.randn(c1 - c0, cols, generator=_gen(seed, f"{tag}/{i}"), dtype=torch.float32,
                    out=out[c0 - r0:c1 - r0])

    if len(jobs) == 1:
        job(jobs[0])
    else:
        with concurrent.futures.ThreadPoolExecutor(min(_DRAW_THREADS, len(jobs))) as ex:
            list(ex.map(job, jobs))
    return out


@dataclasses.dataclass
class Inputs:
    """Everything one (anchor, target) layer pair holds for a workload.

    Storage tensors are CPU tensors in the workload dtype, laid out exactly as
    the compressed cache keeps them in HBM.  Sequence `n_decode` (if present)
    is the prefill sequence.
    """
    w: Workload
    seq_start: List[int]          # first pool row of each sequence
    seq_len: List[int]            # valid tokens of each sequence
    seq_cap: List[int]            # rows reserved for each sequence
    n_decode: int                 # sequences that take a decode query
    K_a: torch.Tensor             # [pool, D]  anchor layer keys
    V_a: torch.Tensor             # [pool, D]  anchor layer values
    K_r: torch.Tensor             # [pool, m]  target layer retained key dims
    V_r: torch.Tensor             # [pool, m]
    W_K: torch.Tensor             # [d_in, d_out]
    W_V: torch.Tensor             # [d_in, d_out]
    q: torch.Tensor               # [n_decode, H_q, d]
    q_prefill: Optional[torch.Tensor]   # [T_q, H_q, d] or None
    q_pos0: int                   # position of the first prefill query

    @property
    def pool_tokens(self) -> int:
        return int(self.K_a.shape[0])

    @property
    def total_decode_tokens(self) -> int:
        return int(sum(self.seq_len[: self.n_decode]))

    def rows(self, b: int) -> slice:
        return slice(self.seq_start[b], self.seq_start[b] + self.seq_len[b])


def generate(w: Workload) -> Inputs:
    if w.n_q_heads % w.n_kv_heads:
        raise ValueError("H_q must be a multiple of H_kv")
    if not 0 <= w.n_retained <= w.D:
        raise ValueError("need 0 <= m <= D")
    lens = draw_lengths(w)
    n_decode = len(lens)
    if w.prefill_len:
        if not 0 < w.prefill_q <= w.prefill_len:
            raise ValueError("need 0 < prefill_q <= prefill_len")
        lens = lens + [int(w.prefill_len)]
    caps = [_round_up(max(x, 1), ROW_ALIGN) for x in lens]
    starts, acc = [], 0
    for c in caps:
        starts.append(acc)
        acc += c
    pool = acc
    D, m = w.D, w.n_retained
    td = w.torch_dtype

    gaps = [(s_ + n_, s_ + c_) for s_, n_, c_ in zip(starts, lens, caps) if c_ > n_]

    def layer_pair(tag):
        """Anchor rows A ~ N(0,1) and the target's retained prefix A @ M1 + 0.1 E1."""
        a_out = torch.empty(pool, D, dtype=td)
        r_out = torch.empty(pool, m, dtype=td)
        M1 = torch.randn(D, m, generator=_gen(w.seed, "M1_" + tag),
                         dtype=torch.float32) / math.sqrt(D) if m else None
        block = _CHUNK_ROWS * _DRAW_THREADS
        for r0 in range(0, pool, block):
            r1 = min(pool, r0 + block)
            a = _draw_rows(r0, r1, D, w.seed, tag + "_a")
            a_out[r0:r1].copy_(a)
            if m:
                e = _draw_rows(r0, r1, m, w.seed, "E1_" + tag)
                e.mul_(0.1)
                e.addmm_(a, M1)                 # A @ M1 + 0.1 E1, in place
                r_out[r0:r1].copy_(e)
        for g0, g1 in gaps:                     # rows no sequence owns stay zero
            a_out[g0:g1] = 0
            r_out[g0:g1] = 0
        return a_out, r_out

    K_a, K_r = layer_pair("K")
    V_a, V_r = layer_pair("V")

    d_in, d_out = w.d_in, w.d_out
    def weight(tag):
        return (torch.randn(d_in, d_out, generator=_gen(w.seed, tag),
                            dtype=torch.float32) / math.sqrt(d_in)).to(td)
    W_K, W_V = weight("W_K"), weight("W_V")

    q = torch.randn(n_decode, w.n_q_heads, w.head_dim,
                    generator=_gen(w.seed, "q"), dtype=torch.float32).to(td)
    q_p, q_pos0 = None, 0
    if w.prefill_len:
        q_p = torch.randn(w.prefill_q, w.n_q_heads, w.head_dim,
                          generator=_gen(w.seed, "q_prefill"),
                          dtype=torch.float32).to(td)
        q_pos0 = w.prefill_len - w.prefill_q
    return Inputs(w, starts, lens, caps, n_decode, K_a, V_a, K_r, V_r,
                  W_K, W_V, q, q_p, q_pos0)


def selector_weights(w: Workload, source_cols: Sequence[int]) -> torch.Tensor:
    """W whose output column c copies predictor-input column source_cols[c].

    Pure 0/1 layout helper for identity-style test cases; exact in any dtype.
    """
    if len(source_cols) != w.d_out:
        raise ValueError("need one source column per output column")
    W = torch.zeros(w.d_in, w.d_out, dtype=w.torch_dtype)
    for c, s in enumerate(source_cols):
        W[int(s), c] = 1.0
    return W


def rope_tables(head_dim: int, n_pos: int, base: float = 10000.0):
    """Angle tables a caller of the rotary-embedding decode passes in: cos, sin
    [n_pos, head_dim / 2] fp32 with angle(p, i) = p * base^(-2 i / head_dim)
    (worked out in float64, stored as float32)."""
    i = torch.arange(head_dim // 2, dtype=torch.float64)
    ang = torch.arange(n_pos, dtype=torch.float64)[:, None] * base ** (-2.0 * i / head_dim)[None, :]
    return torch.cos(ang).to(torch.float32), torch.sin(ang).to(torch.float32)


def window_rows(inp: Inputs, n_sink: int, n_recent: int):
    """Uncompressed rows of the target layer for the first n_sink and the latest
    n_recent positions of every decode sequence: win_k, win_v
    [n_decode, n_sink + n_recent, D].  The first m dims repeat what the
    compressed cache stores for that token; the dropped dims are fresh seeded
    draws (so they differ from anything the predictor would rebuild).  Position
    p sits in row p (p < n_sink) or n_sink + (p - n_sink) % n_recent."""
    w = inp.w
    W_ = n_sink + n_recent
    out = []
    for tag, src in (("win_k", inp.K_r), ("win_v", inp.V_r)):
        win = torch.zeros(inp.n_decode, W_, w.D, dtype=w.torch_dtype)
        for b in range(inp.n_decode):
            L = inp.seq_len[b]
            rows = torch.randn(W_, w.D, generator=_gen(w.seed, f"{tag}_{b}"), dtype=torch.float32)
            for p in list(range(min(n_sink, L))) + list(range(max(n_sink, L - n_recent), L)):
                r = p if p < n_sink else n_sink + (p - n_sink) % n_recent
                win[b, r] = rows[r].to(w.torch_dtype)
                if w.n_retained:
                    win[b, r, :w.n_retained] = src[inp.seq_start[b] + p]
        out.append(win)
    return out[0], out[1]


def mlp_weights(w: Workload, hidden: int):
    """Weights of a one-hidden-layer predictor for workload w: W1 [d_in, hidden] ~
    N(0, 1/sqrt(d_in)), W2 [hidden, d_out] ~ N(0, sqrt(2/hidden)) (keeps the
    rebuilt dims near unit variance behind a ReLU), for keys and for values."""
    out = []
    for tag in ("K", "V"):
        w1 = torch.randn(w.d_in, hidden, generator=_gen(w.seed, "mlp_W1_" + tag),
                         dtype=torch.float32) / math.sqrt(w.d_in)
        w2 = torch.randn(hidden, w.d_out, generator=_gen(w.seed, "mlp_W2_" + tag),
                         dtype=torch.float32) * math.sqrt(2.0 / hidden)
        out += [w1.to(w.torch_dtype), w2.to(w.torch_dtype)]
    return tuple(out)          # W1_K, W2_K, W1_V, W2_V
