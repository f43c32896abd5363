"""ctypes binding over libechokv.so: argument marshalling only.

Function names mirror the C ABI in include/echokv.h.  Tensors are torch tensors
used as device buffers; `stream` defaults to torch's current HIP stream.  There
is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_LIB = None
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libechokv.so")

OK, ERR_NULL, ERR_SHAPE, ERR_DTYPE, ERR_CAPACITY, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP, ERR_STATIC_LIMIT = range(9)
STATIC_SCRATCH_BYTES = 32 << 20
BF16, F32 = 0, 1
FLAG_UNFUSED = 1
FLAG_W_PACKED = 2
FLAG_STAGED = 4
FLAG_ABSORBED = 8
FLAG_ABSORB_V = 16
FLAG_W_AUGMENTED = 32

EXPORTS = ("echokv_status_string", "echokv_cache_append", "echokv_reconstruct",
           "echokv_workspace_bytes", "echokv_decode_attn", "echokv_prefill_attn",
           "echokv_profile_enable", "echokv_profile_read", "echokv_pack_weights",
           "echokv_cache_compress", "echokv_decode_attn_ex", "echokv_window_append",
           "echokv_mlp_workspace_bytes", "echokv_decode_attn_mlp", "echokv_profile_stream_read",
           "echokv_fit_workspace_bytes", "echokv_fit_linear", "echokv_prefill_attn_ex",
           "echokv_decode_attn_static", "echokv_profile_read_channel", "echokv_decode_path",
           "echokv_augmented_weight_elems", "echokv_augment_weights")
ACT_RELU, ACT_SILU = 1, 2
PATH_FUSED, PATH_FUSED_DIRECT, PATH_UNFUSED, PATH_ABSORBED, PATH_ABSORB_V, PATH_RETAINED_ONLY = range(6)


class EchoKVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: status {code} ({status_string(code)})")


class Shape(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("n_retained", C.c_int32), ("dtype", C.c_int32), ("out_dtype", C.c_int32),
                ("softmax_scale", C.c_float), ("flags", C.c_uint32)]


class LayerCacheC(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("width", C.c_int32), ("batch", C.c_int32),
                ("pool_tokens", C.c_int64), ("seq_start", C.POINTER(C.c_int64)),
                ("seq_len", C.POINTER(C.c_int32)), ("seq_cap", C.POINTER(C.c_int32))]


class DecodeExtras(C.Structure):
    _fields_ = [("rope_cos", C.c_void_p), ("rope_sin", C.c_void_p), ("rope_positions", C.c_int32),
                ("n_sink", C.c_int32), ("n_recent", C.c_int32), ("win_k", C.c_void_p),
                ("win_v", C.c_void_p)]


def load() -> C.CDLL:
    """Load libechokv.so (built in-tree by build.build_library)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = os.environ.get("ECHOKV_LIB", LIB_PATH)   # A/B builds of the same ABI
    # The tensors handed to this library live in PyTorch's HIP runtime: bring that copy of the
    # runtime into the process first, so that the library's own dependency resolves to it and
    # kernels are launched in the context that owns the memory.
    import torch  # noqa: F401
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it with "
                           "`python -m paper_2603_22910_amd.build` (needs hipcc); "
                           "there is no CPU fallback")
    lib = C.CDLL(path)
    lib.echokv_status_string.restype = C.c_char_p
    lib.echokv_status_string.argtypes = [C.c_int]
    lib.echokv_workspace_bytes.restype = C.c_size_t
    lib.echokv_workspace_bytes.argtypes = [C.POINTER(Shape), C.c_int32, C.c_int64, C.c_int32]
    lib.echokv_cache_append.restype = C.c_int
    lib.echokv_cache_append.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC), C.c_void_p,
                                        C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
    lib.echokv_reconstruct.restype = C.c_int
    lib.echokv_reconstruct.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                       C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_int32,
                                       C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.echokv_decode_attn.restype = C.c_int
    lib.echokv_decode_attn.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                       C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.echokv_decode_attn_static.restype = C.c_int
    lib.echokv_decode_attn_static.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                              C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.echokv_decode_attn_ex.restype = C.c_int
    lib.echokv_decode_attn_ex.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                          C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(DecodeExtras), C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
    lib.echokv_mlp_workspace_bytes.restype = C.c_size_t
    lib.echokv_mlp_workspace_bytes.argtypes = [C.POINTER(Shape), C.c_int32, C.c_int64, C.c_int32]
    lib.echokv_decode_attn_mlp.restype = C.c_int
    lib.echokv_decode_attn_mlp.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                           C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.echokv_fit_workspace_bytes.restype = C.c_size_t
    lib.echokv_fit_workspace_bytes.argtypes = [C.POINTER(Shape), C.c_int64]
    lib.echokv_fit_linear.restype = C.c_int
    lib.echokv_fit_linear.argtypes = [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_int64, C.c_float,
                                      C.c_int32, C.c_float, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p]
    lib.echokv_window_append.restype = C.c_int
    lib.echokv_window_append.argtypes = [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_void_p,
                                         C.c_void_p, C.POINTER(C.c_int32), C.c_void_p]
    lib.echokv_prefill_attn.restype = C.c_int
    lib.echokv_prefill_attn.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                        C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    lib.echokv_prefill_attn_ex.restype = C.c_int
    lib.echokv_prefill_attn_ex.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                           C.POINTER(LayerCacheC), C.c_void_p, C.c_void_p, C.c_int32,
                                           C.c_void_p, C.c_int32, C.c_int32, C.POINTER(DecodeExtras),
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.echokv_cache_compress.restype = C.c_int
    lib.echokv_cache_compress.argtypes = [C.POINTER(Shape), C.POINTER(LayerCacheC),
                                          C.POINTER(LayerCacheC), C.c_void_p]
    lib.echokv_pack_weights.restype = C.c_int
    lib.echokv_pack_weights.argtypes = [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p]
    lib.echokv_augmented_weight_elems.restype = C.c_size_t
    lib.echokv_augmented_weight_elems.argtypes = [C.POINTER(Shape)]
    lib.echokv_augment_weights.restype = C.c_int
    lib.echokv_augment_weights.argtypes = [C.POINTER(Shape), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p]
    lib.echokv_profile_enable.restype = C.c_int
    lib.echokv_profile_enable.argtypes = [C.c_int]
    lib.echokv_profile_read.restype = C.c_int
    lib.echokv_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.echokv_decode_path.restype = C.c_int
    lib.echokv_decode_path.argtypes = [C.POINTER(Shape), C.POINTER(C.c_int32)]
    lib.echokv_profile_read_channel.restype = C.c_int
    lib.echokv_profile_read_channel.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.echokv_profile_stream_read.restype = C.c_int
    lib.echokv_profile_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.POINTER(C.c_double)]
    _LIB = lib
    return lib


def status_string(code: int) -> str:
    return load().echokv_status_string(int(code)).decode()


def make_shape(n_q_heads: int, n_kv_heads: int, head_dim: int, n_retained: int, dtype: str,
               out_dtype: Optional[str] = None, softmax_scale: float = 0.0,
               flags: int = 0) -> Shape:
    code = {"bf16": BF16, "f32": F32}
    return Shape(n_q_heads, n_kv_heads, head_dim, n_retained, code[dtype],
                 code[out_dtype or dtype], float(softmax_scale), int(flags))


class LayerCache:
    """One layer's K/V pool plus the host-side sequence table.

    k, v: torch tensors [pool_tokens, width] on the GPU (or None when width == 0).
    The sequence arrays live in NumPy so the C side can read and update them.
    """

    def __init__(self, k, v, width: int, pool_tokens: int, seq_start: Sequence[int],
                 seq_len: Sequence[int], seq_cap: Sequence[int]):
        self.k, self.v = k, v
        self.width = int(width)
        self.pool_tokens = int(pool_tokens)
        self.seq_start = np.ascontiguousarray(seq_start, dtype=np.int64)
        self.seq_len = np.ascontiguousarray(seq_len, dtype=np.int32)
        self.seq_cap = np.ascontiguousarray(seq_cap, dtype=np.int32)

    @property
    def batch(self) -> int:
        return int(self.seq_start.shape[0])

    def view(self, first: int, count: int) -> "LayerCache":
        """The same pool restricted to sequences [first, first+count) (shares the arrays)."""
        c = LayerCache.__new__(LayerCache)
        c.k, c.v, c.width, c.pool_tokens = self.k, self.v, self.width, self.pool_tokens
        c.seq_start = self.seq_start[first:first + count]
        c.seq_len = self.seq_len[first:first + count]
        c.seq_cap = self.seq_cap[first:first + count]
        return c

    def as_c(self) -> LayerCacheC:
        # built once per (tensors, arrays): a decode loop calls this three times a step
        key = (id(self.k), id(self.v), id(self.seq_start), id(self.seq_len), id(self.seq_cap),
               self.width, self.pool_tokens)
        if getattr(self, "_c_key", None) != key:
            self._c = LayerCacheC(
                _ptr(self.k), _ptr(self.v), self.width, self.batch, self.pool_tokens,
                self.seq_start.ctypes.data_as(C.POINTER(C.c_int64)),
                self.seq_len.ctypes.data_as(C.POINTER(C.c_int32)),
                self.seq_cap.ctypes.data_as(C.POINTER(C.c_int32)))
            self._c_key = key
        return self._c


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(rc: int, where: str):
    if rc != OK:
        raise EchoKVError(rc, where)


def workspace_bytes(shape: Shape, batch: int, total_tokens: int, max_q: int = 0) -> int:
    return int(load().echokv_workspace_bytes(C.byref(shape), batch, total_tokens, max_q))


def cache_append(shape: Shape, dst: LayerCache, k_new, v_new, n_new: Sequence[int], stream=None):
    n = np.ascontiguousarray(n_new, dtype=np.int32)
    c = dst.as_c()
    _check(load().echokv_cache_append(C.byref(shape), C.byref(c), _ptr(k_new), _ptr(v_new),
                                      n.ctypes.data_as(C.POINTER(C.c_int32)), _stream(stream)),
           "echokv_cache_append")


def cache_compress(shape: Shape, full: LayerCache, dst: LayerCache, stream=None):
    f, d = full.as_c(), dst.as_c()
    _check(load().echokv_cache_compress(C.byref(shape), C.byref(f), C.byref(d), _stream(stream)),
           "echokv_cache_compress")


def reconstruct(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, seq: int,
                tok_begin: int, tok_end: int, k_out, v_out, stream=None):
    a, t = anchor.as_c(), target.as_c()
    _check(load().echokv_reconstruct(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k), _ptr(w_v),
                                     seq, tok_begin, tok_end, _ptr(k_out), _ptr(v_out),
                                     _stream(stream)), "echokv_reconstruct")


def decode_attn(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, q, out,
                lse_out, workspace, stream=None):
    a, t = anchor.as_c(), target.as_c()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().echokv_decode_attn(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k), _ptr(w_v),
                                     _ptr(q), _ptr(out), _ptr(lse_out), _ptr(workspace), nbytes,
                                     _stream(stream)), "echokv_decode_attn")


def decode_path(shape: Shape) -> int:
    """One of PATH_*: the kernels echokv_decode_attn runs for this shape and its flags."""
    out = C.c_int32(-1)
    _check(load().echokv_decode_path(C.byref(shape), C.byref(out)), "echokv_decode_path")
    return int(out.value)


def decode_attn_static(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, q, out,
                       lse_out, stream=None):
    """echokv_decode_attn on the library's fixed scratch: no workspace, nothing allocated."""
    a, t = anchor.as_c(), target.as_c()
    _check(load().echokv_decode_attn_static(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k),
                                            _ptr(w_v), _ptr(q), _ptr(out), _ptr(lse_out),
                                            _stream(stream)), "echokv_decode_attn_static")


def decode_attn_ex(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, q, out,
                   lse_out, workspace, rope=None, window=None, stream=None):
    """rope = (cos, sin) device fp32 [positions, d/2]; window = (win_k, win_v, n_sink, n_recent)."""
    a, t = anchor.as_c(), target.as_c()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ex = DecodeExtras()
    if rope is not None:
        ex.rope_cos, ex.rope_sin, ex.rope_positions = _ptr(rope[0]), _ptr(rope[1]), int(rope[0].shape[0])
    if window is not None:
        ex.win_k, ex.win_v, ex.n_sink, ex.n_recent = _ptr(window[0]), _ptr(window[1]), int(window[2]), int(window[3])
    _check(load().echokv_decode_attn_ex(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k), _ptr(w_v),
                                        _ptr(q), C.byref(ex), _ptr(out), _ptr(lse_out),
                                        _ptr(workspace), nbytes, _stream(stream)),
           "echokv_decode_attn_ex")


def mlp_workspace_bytes(shape: Shape, batch: int, total_tokens: int, hidden: int) -> int:
    return int(load().echokv_mlp_workspace_bytes(C.byref(shape), int(batch), int(total_tokens), int(hidden)))


def decode_attn_mlp(shape: Shape, anchor: LayerCache, target: LayerCache, w1_k, w2_k, w1_v, w2_v,
                    hidden: int, activation: int, q, out, lse_out, workspace, stream=None):
    a, t = anchor.as_c(), target.as_c()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().echokv_decode_attn_mlp(C.byref(shape), C.byref(a), C.byref(t), _ptr(w1_k), _ptr(w2_k),
                                         _ptr(w1_v), _ptr(w2_v), int(hidden), int(activation), _ptr(q),
                                         _ptr(out), _ptr(lse_out), _ptr(workspace), nbytes,
                                         _stream(stream)), "echokv_decode_attn_mlp")


def fit_workspace_bytes(shape: Shape, n_rows: int) -> int:
    return int(load().echokv_fit_workspace_bytes(C.byref(shape), int(n_rows)))


def fit_linear(shape: Shape, anchor_rows, target_rows, n_rows: int, w_out, workspace, ridge: float = 0.0,
               max_iters: int = 200, tol: float = 1e-5, stream=None):
    """Returns (iterations, relative residual of the normal equations)."""
    it, res = C.c_int32(0), C.c_float(0.0)
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().echokv_fit_linear(C.byref(shape), _ptr(anchor_rows), _ptr(target_rows), int(n_rows),
                                    float(ridge), int(max_iters), float(tol), _ptr(w_out), _ptr(workspace),
                                    nbytes, C.byref(it), C.byref(res), _stream(stream)), "echokv_fit_linear")
    return int(it.value), float(res.value)


def window_append(shape: Shape, win_k, win_v, n_sink: int, n_recent: int, seq_len_before, k_new,
                  v_new, n_new, stream=None):
    before = np.ascontiguousarray(seq_len_before, dtype=np.int32)
    nn = np.ascontiguousarray(n_new, dtype=np.int32)
    _check(load().echokv_window_append(C.byref(shape), _ptr(win_k), _ptr(win_v), int(n_sink),
                                       int(n_recent), len(nn),
                                       before.ctypes.data_as(C.POINTER(C.c_int32)), _ptr(k_new),
                                       _ptr(v_new), nn.ctypes.data_as(C.POINTER(C.c_int32)),
                                       _stream(stream)), "echokv_window_append")


def prefill_attn(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, seq: int, q,
                 T_q: int, q_pos0: int, out, lse_out, workspace, stream=None):
    a, t = anchor.as_c(), target.as_c()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().echokv_prefill_attn(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k), _ptr(w_v),
                                      seq, _ptr(q), T_q, q_pos0, _ptr(out), _ptr(lse_out),
                                      _ptr(workspace), nbytes, _stream(stream)),
           "echokv_prefill_attn")


def prefill_attn_ex(shape: Shape, anchor: LayerCache, target: LayerCache, w_k, w_v, seq: int, q,
                    T_q: int, q_pos0: int, out, lse_out, workspace, rope=None, window=None, stream=None):
    """rope = (cos, sin) device fp32 [positions, d/2]; window is refused by the library."""
    a, t = anchor.as_c(), target.as_c()
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    ex = DecodeExtras()
    if rope is not None:
        ex.rope_cos, ex.rope_sin, ex.rope_positions = _ptr(rope[0]), _ptr(rope[1]), int(rope[0].shape[0])
    if window is not None:
        ex.win_k, ex.win_v, ex.n_sink, ex.n_recent = _ptr(window[0]), _ptr(window[1]), int(window[2]), int(window[3])
    _check(load().echokv_prefill_attn_ex(C.byref(shape), C.byref(a), C.byref(t), _ptr(w_k), _ptr(w_v),
                                         seq, _ptr(q), T_q, q_pos0, C.byref(ex), _ptr(out),
                                         _ptr(lse_out), _ptr(workspace), nbytes, _stream(stream)),
           "echokv_prefill_attn_ex")


def pack_weights(shape: Shape, w, w_packed, stream=None):
    _check(load().echokv_pack_weights(C.byref(shape), _ptr(w), _ptr(w_packed), _stream(stream)),
           "echokv_pack_weights")


def augmented_weight_elems(shape: Shape) -> int:
    return int(load().echokv_augmented_weight_elems(C.byref(shape)))


def augment_weights(shape: Shape, w_k, w_v, w_k_aug, w_v_aug, stream=None):
    _check(load().echokv_augment_weights(C.byref(shape), _ptr(w_k), _ptr(w_v), _ptr(w_k_aug), _ptr(w_v_aug),
                                         _stream(stream)), "echokv_augment_weights")


def profile_stream_read(buf, repeats: int = 5) -> float:
    """GB/s a plain streaming-read kernel reaches over the tensor `buf`."""
    out = C.c_double(0.0)
    _check(load().echokv_profile_stream_read(_ptr(buf), buf.numel() * buf.element_size(), int(repeats),
                                             C.byref(out)), "echokv_profile_stream_read")
    return float(out.value)


def profile_enable(on: bool):
    _check(load().echokv_profile_enable(1 if on else 0), "echokv_profile_enable")


def profile_read(channel: int = 0):
    """(total milliseconds, launches) since the last read.  Channel 0: the dominant decode
    kernel(s); 1: a prefill chunk's predictor product; 2: its attention kernel."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(load().echokv_profile_read_channel(int(channel), C.byref(ms), C.byref(n)),
           "echokv_profile_read_channel")
    return float(ms.value), int(n.value)
