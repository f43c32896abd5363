"""Device-side harness: puts a synthetic workload into HBM in the compressed
cache layout and drives the C ABI.  PyTorch is used for device memory, streams
and events only; no arithmetic of the method happens here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as ek
from .synth import Inputs


class DeviceWorkload:
    def __init__(self, inp: Inputs, out_dtype: Optional[str] = None, flags: int = 0,
                 softmax_scale: float = 0.0, device: str = "cuda:0"):
        if not torch.cuda.is_available():
            raise RuntimeError("an MI355X is required: libechokv has no CPU path")
        ek.load()
        w = inp.w
        self.inp, self.w = inp, w
        self.dev = torch.device(device)
        self.out_dtype = out_dtype or w.dtype
        self.shape = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_retained, w.dtype,
                                   self.out_dtype, softmax_scale, flags)
        up = lambda t: t.to(self.dev, non_blocking=False).contiguous()
        self.K_a, self.V_a = up(inp.K_a), up(inp.V_a)
        self.K_r = up(inp.K_r) if w.n_retained else None
        self.V_r = up(inp.V_r) if w.n_retained else None
        self.W_K = up(inp.W_K) if w.d_out else None
        self.W_V = up(inp.W_V) if w.d_out else None
        self.q = up(inp.q)
        self.q_prefill = up(inp.q_prefill) if inp.q_prefill is not None else None
        self.anchor_all = ek.LayerCache(self.K_a, self.V_a, w.D, inp.pool_tokens, inp.seq_start,
                                        inp.seq_len, inp.seq_cap)
        self.target_all = ek.LayerCache(self.K_r, self.V_r, w.n_retained, inp.pool_tokens,
                                        inp.seq_start, inp.seq_len, inp.seq_cap)
        self.anchor = self.anchor_all.view(0, inp.n_decode)
        self.target = self.target_all.view(0, inp.n_decode)
        tdt = {"bf16": torch.bfloat16, "f32": torch.float32}[self.out_dtype]
        self.out = torch.empty(inp.n_decode, w.n_q_heads, w.head_dim, dtype=tdt, device=self.dev)
        self.lse = torch.empty(inp.n_decode, w.n_q_heads, dtype=torch.float32, device=self.dev)
        need = ek.workspace_bytes(self.shape, inp.n_decode, inp.total_decode_tokens, 0)
        self.out_prefill = self.lse_prefill = None
        if self.q_prefill is not None:
            T_q = int(self.q_prefill.shape[0])
            need = max(need, ek.workspace_bytes(self.shape, 1, inp.seq_len[-1], T_q))
            self.out_prefill = torch.empty(T_q, w.n_q_heads, w.head_dim, dtype=tdt, device=self.dev)
            self.lse_prefill = torch.empty(T_q, w.n_q_heads, dtype=torch.float32, device=self.dev)
        if need == 0:
            raise RuntimeError("echokv_workspace_bytes rejected the shape")
        self.workspace = torch.empty(need, dtype=torch.uint8, device=self.dev)

    def set_flags(self, flags: int):
        self.shape.flags = flags

    def pack_weights(self):
        """Lay W_K / W_V out once as [d_out, d_in] and make decode() use them."""
        if self.W_K is None:
            return
        self.W_K_packed = torch.empty(self.w.d_out, self.w.d_in, dtype=self.W_K.dtype, device=self.dev)
        self.W_V_packed = torch.empty_like(self.W_K_packed)
        ek.pack_weights(self.shape, self.W_K, self.W_K_packed)
        ek.pack_weights(self.shape, self.W_V, self.W_V_packed)
        self.shape.flags |= ek.FLAG_W_PACKED

    def decode(self, stream=None):
        packed = bool(self.shape.flags & ek.FLAG_W_PACKED)
        wk, wv = (self.W_K_packed, self.W_V_packed) if packed else (self.W_K, self.W_V)
        ek.decode_attn(self.shape, self.anchor, self.target, wk, wv, self.q, self.out,
                       self.lse, self.workspace, stream)
        return self.out, self.lse

    def decode_ex(self, rope=None, window=None, stream=None):
        """rope = (cos, sin) host or device fp32 tables; window = (win_k, win_v, n_sink, n_recent)."""
        if rope is not None:
            rope = tuple(t.to(self.dev).contiguous() for t in rope)
        if window is not None:
            window = (window[0].to(self.dev).contiguous(), window[1].to(self.dev).contiguous(),
                      window[2], window[3])
        self._keep = (rope, window)          # keep the device copies alive until the stream is done
        ek.decode_attn_ex(self.shape, self.anchor, self.target, self.W_K, self.W_V, self.q, self.out,
                          self.lse, self.workspace, rope, window, stream)
        return self.out, self.lse

    def decode_mlp(self, weights, hidden: int, activation: int, stream=None):
        """weights = (W1_K, W2_K, W1_V, W2_V) host or device tensors."""
        wts = tuple(t.to(self.dev).contiguous() for t in weights)
        need = ek.mlp_workspace_bytes(self.shape, self.inp.n_decode, self.inp.total_decode_tokens, hidden)
        if need == 0:
            raise RuntimeError("echokv_mlp_workspace_bytes rejected the shape")
        if getattr(self, "_mlp_ws", None) is None or self._mlp_ws.numel() < need:
            self._mlp_ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        self._keep = wts
        ek.decode_attn_mlp(self.shape, self.anchor, self.target, wts[0], wts[1], wts[2], wts[3], hidden,
                           activation, self.q, self.out, self.lse, self._mlp_ws, stream)
        return self.out, self.lse

    def prefill(self, stream=None):
        saved = self.shape.flags
        self.shape.flags = saved & ~ek.FLAG_W_PACKED      # prefill takes row-major weights
        try:
            return self._prefill(stream)
        finally:
            self.shape.flags = saved

    def _prefill(self, stream=None, rope=None):
        seq = self.inp.n_decode
        T_q = int(self.q_prefill.shape[0])
        if rope is None:
            ek.prefill_attn(self.shape, self.anchor_all, self.target_all, self.W_K, self.W_V, seq,
                            self.q_prefill, T_q, self.inp.q_pos0, self.out_prefill, self.lse_prefill,
                            self.workspace, stream)
        else:
            ek.prefill_attn_ex(self.shape, self.anchor_all, self.target_all, self.W_K, self.W_V, seq,
                               self.q_prefill, T_q, self.inp.q_pos0, self.out_prefill,
                               self.lse_prefill, self.workspace, rope=rope, stream=stream)
        return self.out_prefill, self.lse_prefill

    def prefill_ex(self, rope, stream=None):
        """rope = (cos, sin) host or device fp32 tables [positions, d/2]."""
        rope = tuple(t.to(self.dev).contiguous() for t in rope)
        self._keep = rope
        saved = self.shape.flags
        self.shape.flags = saved & ~ek.FLAG_W_PACKED
        try:
            return self._prefill(stream, rope)
        finally:
            self.shape.flags = saved

    def reconstruct(self, seq: int, tok_begin: int, tok_end: int, stream=None):
        w = self.w
        n = tok_end - tok_begin
        k_out = torch.empty(n, w.D, dtype=w.torch_dtype, device=self.dev)
        v_out = torch.empty(n, w.D, dtype=w.torch_dtype, device=self.dev)
        ek.reconstruct(self.shape, self.anchor_all, self.target_all, self.W_K, self.W_V, seq,
                       tok_begin, tok_end, k_out, v_out, stream)
        return k_out, v_out


def error_metrics(got: np.ndarray, ref: np.ndarray):
    """(max abs error, relative L2 error over the whole tensor)."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
