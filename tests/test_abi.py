"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2603_22910_amd import binding as ek

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x100000  # non-null stand-in for a device pointer; never dereferenced on these paths


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ek.LIB_PATH):
        from paper_2603_22910_amd import build
        build.build_library()
    return ek.load()


def test_exports_match_header(lib):
    hdr = open(os.path.join(ROOT, "include", "echokv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(echokv_[a-z_]+)\s*\(", hdr))
    assert declared == set(ek.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header compiles as strict C99 and as C++, and a C program that
    names every declared entry point links against the built library (no compute call is made)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    hdr = open(os.path.join(ROOT, "include", "echokv.h")).read()
    names = sorted(set(re.findall(r"\b(echokv_[a-z_]+)\s*\(", re.sub(r"/\*.*?\*/", "", hdr, flags=re.S))))
    src = tmp_path / "use.c"
    src.write_text('#include "echokv.h"\n#include <stdio.h>\nint main(void) {\n  const void *fn[] = {\n'
                   + "".join(f"    (const void *)(size_t)&{n},\n" for n in names)
                   + '  };\n  printf("%d %s\\n", (int)(sizeof fn / sizeof fn[0]), echokv_status_string(ECHOKV_OK));\n'
                     "  return 0;\n}\n")
    inc = os.path.join(ROOT, "include")
    libdir = os.path.join(ROOT, "paper_2603_22910_amd")
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", inc, "-c", str(src),
                    "-o", str(tmp_path / "use.o")], check=True, capture_output=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-I", inc, "-x", "c++", "-c", str(src),
                    "-o", str(tmp_path / "use_cpp.o")], check=True, capture_output=True)
    exe = tmp_path / "use"
    subprocess.run(["gcc", str(tmp_path / "use.o"), "-o", str(exe), f"-L{libdir}", "-l:libechokv.so",
                    f"-Wl,-rpath,{libdir}"], check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out == [str(len(names)), "ok"]


def test_status_strings(lib):
    seen = {ek.status_string(c) for c in range(9)}
    assert len(seen) == 9 and ek.status_string(0) == "ok"
    assert ek.status_string(99) == "unknown status"


def caches(D=512, m=256, lens=(100,), caps=None, pool=None):
    caps = caps or [256] * len(lens)
    starts = np.cumsum([0] + list(caps[:-1]))
    pool = pool or int(sum(caps))
    a = ek.LayerCache(FAKE, FAKE, D, pool, starts, lens, caps)
    t = ek.LayerCache(FAKE if m else None, FAKE if m else None, m, pool, starts, lens, caps)
    return a, t


def code(fn, *args, **kw):
    try:
        fn(*args, **kw)
    except ek.EchoKVError as e:
        return e.code
    return ek.OK


def test_shape_validation(lib):
    a, t = caches()
    ok = ek.make_shape(8, 8, 64, 256, "f32")
    big = 1 << 30
    args = (a, t, FAKE, FAKE, FAKE, FAKE, None, FAKE)
    for bad, want in [
        (ek.make_shape(8, 3, 64, 256, "f32"), ek.ERR_SHAPE),          # H_q % H_kv
        (ek.make_shape(8, 8, 64, 576, "f32"), ek.ERR_SHAPE),          # m > D
        (ek.make_shape(8, 8, 64, -64, "f32"), ek.ERR_SHAPE),
        (ek.make_shape(8, 8, 64, 96, "f32"), ek.ERR_UNSUPPORTED),     # m % d
        (ek.make_shape(8, 8, 48, 0, "f32"), ek.ERR_UNSUPPORTED),      # head_dim
        (ek.make_shape(0, 8, 64, 256, "f32"), ek.ERR_SHAPE),
    ]:
        assert ek.workspace_bytes(bad, 1, 100, 1) == 0
        assert code(ek.decode_attn, bad, *args[:-1], _Ws(big), stream=0) == want
    bad_dtype = ek.make_shape(8, 8, 64, 256, "f32"); bad_dtype.dtype = 7
    assert code(ek.decode_attn, bad_dtype, *args[:-1], _Ws(big), stream=0) == ek.ERR_DTYPE
    assert ek.workspace_bytes(ok, 1, 100, 1) > 0
    assert ek.workspace_bytes(ok, 0, 100, 1) == 0
    assert ek.workspace_bytes(ok, 1, 100, -1) == 0


def test_workspace_covers_a_prefill_chunk_only_when_asked():
    sh = ek.make_shape(32, 8, 128, 128, "bf16")
    dec = ek.workspace_bytes(sh, 1, 20000, 0)
    one = ek.workspace_bytes(sh, 1, 20000, 1)
    short = ek.workspace_bytes(sh, 1, 20000, 500)
    long_ = ek.workspace_bytes(sh, 1, 20000, 8192)
    assert 0 < dec <= one <= short
    # a short chunk in front of a long context is split over the keys: room for 8 shares of
    # (d + 2) fp32 words per query and head on top of what one query needs
    assert short - one >= 499 * 32 * 8 * 130 * 4 * 0.9
    # chunks of 1024 queries and more are not split, but a caller may still pass shorter ones
    assert long_ - one >= 1023 * 32 * 8 * 130 * 4 * 0.9
    # a prefill call checks the size it needs for its own chunk: a decode-sized workspace is refused
    a = ek.LayerCache(FAKE, FAKE, 1024, 32768, [0], [20000], [32768])
    t = ek.LayerCache(FAKE, FAKE, 128, 32768, [0], [20000], [32768])
    args = (sh, a, t, FAKE, FAKE, 0, FAKE, 500, 19500, FAKE, None)
    assert code(ek.prefill_attn, *args, _Ws(dec), stream=0) == ek.ERR_WORKSPACE
    assert code(ek.prefill_attn, *args, _Ws(short - 256), stream=0) == ek.ERR_WORKSPACE


class _Ws:
    """Workspace stand-in with a fake pointer and a claimed size."""
    def __init__(self, nbytes, ptr=FAKE):
        self._n, self._p = nbytes, ptr
    def numel(self): return self._n
    def element_size(self): return 1
    def data_ptr(self): return self._p


def test_decode_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    a, t = caches()
    big = _Ws(1 << 30)
    assert code(ek.decode_attn, sh, a, t, None, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_NULL
    assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, None, FAKE, None, big, stream=0) == ek.ERR_NULL
    assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, FAKE, None, None, big, stream=0) == ek.ERR_NULL
    assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, FAKE, FAKE, None, None, stream=0) == ek.ERR_WORKSPACE
    assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, FAKE, FAKE, None, _Ws(16), stream=0) == ek.ERR_WORKSPACE
    assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, FAKE, FAKE, None, _Ws(1 << 30, FAKE + 8),
                stream=0) == ek.ERR_WORKSPACE                       # misaligned
    # anchor / target disagree
    a2, t2 = caches(lens=(100,)); t2.seq_len[0] = 99
    assert code(ek.decode_attn, sh, a2, t2, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    a3, t3 = caches(m=128)                                          # target width != m
    assert code(ek.decode_attn, sh, a3, t3, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    a4, t4 = caches(lens=(0,))                                      # empty sequence
    assert code(ek.decode_attn, sh, a4, t4, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    a5, t5 = caches(lens=(300,), caps=[256])                        # len > cap
    assert code(ek.decode_attn, sh, a5, t5, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    a6, t6 = caches(lens=(10,), caps=[256], pool=128)               # cap past the pool
    assert code(ek.decode_attn, sh, a6, t6, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    a7, t7 = caches(); a7.k = None
    assert code(ek.decode_attn, sh, a7, t7, FAKE, FAKE, FAKE, FAKE, None, big, stream=0) == ek.ERR_NULL


def test_full_retention_needs_no_weights_but_others_do(lib):
    sh_full = ek.make_shape(8, 8, 64, 512, "f32")
    a, t = caches(m=512)
    # No weights are needed: the call gets past the weight check and is stopped by the next one, the
    # workspace size.  (Nothing here may reach a launch: these tests hand the library made-up
    # addresses, and on a machine with a GPU a launch would read them.)
    assert code(ek.decode_attn, sh_full, a, t, None, None, FAKE, FAKE, None, _Ws(16), stream=0) == ek.ERR_WORKSPACE
    sh_part = ek.make_shape(8, 8, 64, 256, "f32")
    a2, t2 = caches(m=256)
    assert code(ek.decode_attn, sh_part, a2, t2, None, None, FAKE, FAKE, None, _Ws(16), stream=0) == ek.ERR_NULL


def test_append_errors_leave_lengths_untouched(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    a, t = caches(lens=(250, 10), caps=[256, 256])
    before = t.seq_len.copy()
    assert code(ek.cache_append, sh, t, FAKE, FAKE, [7, 1], stream=0) == ek.ERR_CAPACITY
    assert np.array_equal(t.seq_len, before)
    assert code(ek.cache_append, sh, t, FAKE, FAKE, [-1, 1], stream=0) == ek.ERR_SHAPE
    assert code(ek.cache_append, sh, t, None, FAKE, [1, 1], stream=0) == ek.ERR_NULL
    assert np.array_equal(t.seq_len, before)
    odd = ek.LayerCache(FAKE, FAKE, 128, 512, [0, 256], [1, 1], [256, 256])  # neither D nor m
    assert code(ek.cache_append, sh, odd, FAKE, FAKE, [1, 1], stream=0) == ek.ERR_SHAPE
    # zero new tokens: nothing to launch, succeeds without a device
    assert code(ek.cache_append, sh, t, None, None, [0, 0], stream=0) == ek.OK
    assert np.array_equal(t.seq_len, before)


def test_reconstruct_and_prefill_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    a, t = caches(lens=(100,))
    assert code(ek.reconstruct, sh, a, t, FAKE, FAKE, 1, 0, 10, FAKE, FAKE, stream=0) == ek.ERR_SHAPE
    assert code(ek.reconstruct, sh, a, t, FAKE, FAKE, 0, 5, 101, FAKE, FAKE, stream=0) == ek.ERR_SHAPE
    assert code(ek.reconstruct, sh, a, t, FAKE, FAKE, 0, 7, 5, FAKE, FAKE, stream=0) == ek.ERR_SHAPE
    assert code(ek.reconstruct, sh, a, t, FAKE, None, 0, 0, 10, FAKE, FAKE, stream=0) == ek.ERR_NULL
    assert code(ek.reconstruct, sh, a, t, FAKE, FAKE, 0, 0, 10, None, FAKE, stream=0) == ek.ERR_NULL
    assert code(ek.reconstruct, sh, a, t, FAKE, FAKE, 0, 10, 10, FAKE, FAKE, stream=0) == ek.OK
    big = _Ws(1 << 30)
    pf = lambda seq, T_q, q0, ws=big: code(ek.prefill_attn, sh, a, t, FAKE, FAKE, seq, FAKE, T_q, q0,
                                           FAKE, None, ws, stream=0)
    assert pf(0, 50, 60) == ek.ERR_SHAPE          # chunk not in the cache yet
    assert pf(0, 0, 0) == ek.ERR_SHAPE
    assert pf(2, 10, 0) == ek.ERR_SHAPE
    assert pf(0, 10, 0, _Ws(8)) == ek.ERR_WORKSPACE


def test_compress_and_pack_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    full = ek.LayerCache(FAKE, FAKE, 512, 512, [0, 256], [100, 10], [256, 256])
    dst = ek.LayerCache(FAKE, FAKE, 256, 512, [0, 256], [0, 0], [64, 256])
    assert code(ek.cache_compress, sh, full, dst, stream=0) == ek.ERR_CAPACITY
    assert list(dst.seq_len) == [0, 0]
    wrong = ek.LayerCache(FAKE, FAKE, 128, 512, [0, 256], [0, 0], [256, 256])
    assert code(ek.cache_compress, sh, full, wrong, stream=0) == ek.ERR_SHAPE
    one = ek.LayerCache(FAKE, FAKE, 256, 512, [0], [0], [256])
    assert code(ek.cache_compress, sh, full, one, stream=0) == ek.ERR_SHAPE
    assert code(ek.pack_weights, sh, None, FAKE, stream=0) == ek.ERR_NULL
    assert code(ek.pack_weights, sh, FAKE, FAKE, stream=0) == ek.ERR_SHAPE      # in place
    full_ret = ek.make_shape(8, 8, 64, 512, "f32")
    assert code(ek.pack_weights, full_ret, None, None, stream=0) == ek.OK      # nothing to pack


def test_augmented_weights_argument_rules():
    split = ek.make_shape(32, 8, 128, 64, "bf16")                     # m = 64 cuts head 0 in two: r = 64
    whole = ek.make_shape(32, 8, 128, 128, "bf16")
    assert ek.augmented_weight_elems(split) == (1024 + 64) * (1024 - 64 + 64)
    assert ek.augmented_weight_elems(whole) == (1024 + 128) * (1024 - 128)        # r = 0: the plain size
    assert ek.augmented_weight_elems(ek.make_shape(8, 3, 64, 256, "f32")) == 0
    assert code(ek.augment_weights, split, None, FAKE, FAKE, FAKE, stream=0) == ek.ERR_NULL
    assert code(ek.augment_weights, split, FAKE, FAKE, FAKE, FAKE, stream=0) == ek.ERR_SHAPE     # in place
    assert code(ek.augment_weights, ek.make_shape(8, 8, 64, 512, "f32"), None, None, None, None, stream=0) == ek.OK
    # entry points that do not take extended weights say so
    a = ek.LayerCache(FAKE, FAKE, 1024, 512, [0], [100], [256])
    t = ek.LayerCache(FAKE, FAKE, 64, 512, [0], [100], [256])
    aug = ek.make_shape(32, 8, 128, 64, "bf16"); aug.flags = ek.FLAG_W_AUGMENTED
    assert code(ek.reconstruct, aug, a, t, FAKE, FAKE, 0, 0, 10, FAKE, FAKE, stream=0) == ek.ERR_UNSUPPORTED
    for mode in (ek.FLAG_ABSORBED, ek.FLAG_ABSORB_V):
        sh = ek.make_shape(32, 8, 128, 64, "bf16"); sh.flags = ek.FLAG_W_AUGMENTED | mode
        assert code(ek.decode_attn, sh, a, t, FAKE, FAKE, FAKE, FAKE, None, _Ws(1 << 30), stream=0) == ek.ERR_UNSUPPORTED


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(ek, "_LIB", None)
    monkeypatch.setattr(ek, "LIB_PATH", str(tmp_path / "libechokv.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        ek.load()


class _Tbl:
    """Device-table stand-in: fake pointer, claimed number of rows."""
    def __init__(self, rows, ptr=FAKE):
        self.shape = (rows, 32); self._p = ptr
    def data_ptr(self): return self._p


def test_decode_extras_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    a, t = caches(lens=(100,))
    big = _Ws(1 << 30)
    base = (sh, a, t, FAKE, FAKE, FAKE, FAKE, None, big)
    # tables shorter than the longest sequence
    assert code(ek.decode_attn_ex, *base, rope=(_Tbl(99), _Tbl(99)), stream=0) == ek.ERR_SHAPE
    # one table / one window buffer missing
    half = ek.DecodeExtras(); half.rope_cos = FAKE; half.rope_positions = 200
    a_c, t_c = a.as_c(), t.as_c()
    import ctypes as C
    def raw(ex):
        return lib.echokv_decode_attn_ex(C.byref(sh), C.byref(a_c), C.byref(t_c), FAKE, FAKE, FAKE,
                                         C.byref(ex), FAKE, None, FAKE, 1 << 30, None)
    assert raw(half) == ek.ERR_NULL
    halfw = ek.DecodeExtras(); halfw.win_k = FAKE; halfw.n_sink = 4; halfw.n_recent = 128
    assert raw(halfw) == ek.ERR_NULL
    # window sizes
    assert code(ek.decode_attn_ex, *base, window=(_Tbl(1), _Tbl(1), -1, 128), stream=0) == ek.ERR_SHAPE
    assert code(ek.decode_attn_ex, *base, window=(_Tbl(1), _Tbl(1), 0, 0), stream=0) == ek.ERR_SHAPE
    # the absorbed mode cannot take a rotation between reconstruction and the dot product
    shb = ek.make_shape(8, 8, 64, 256, "bf16", flags=ek.FLAG_ABSORBED)
    assert code(ek.decode_attn_ex, shb, a, t, FAKE, FAKE, FAKE, FAKE, None, big,
                rope=(_Tbl(200), _Tbl(200)), stream=0) == ek.ERR_UNSUPPORTED


def test_prefill_extras_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    a, t = caches(lens=(100,))
    big = _Ws(1 << 30)
    base = (sh, a, t, FAKE, FAKE, 0, FAKE, 10, 90, FAKE, None, big)
    # tables shorter than the chunk's last position
    assert code(ek.prefill_attn_ex, *base, rope=(_Tbl(99), _Tbl(99)), stream=0) == ek.ERR_SHAPE
    # a prefill chunk reads the compressed cache only
    assert code(ek.prefill_attn_ex, *base, window=(_Tbl(1), _Tbl(1), 4, 128), stream=0) == ek.ERR_UNSUPPORTED
    # one table missing
    import ctypes as C
    half = ek.DecodeExtras(); half.rope_cos = FAKE; half.rope_positions = 200
    a_c, t_c = a.as_c(), t.as_c()
    assert lib.echokv_prefill_attn_ex(C.byref(sh), C.byref(a_c), C.byref(t_c), FAKE, FAKE, 0, FAKE, 10, 90,
                                      C.byref(half), FAKE, None, FAKE, 1 << 30, None) == ek.ERR_NULL


def test_window_append_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "f32")
    assert code(ek.window_append, sh, None, FAKE, 4, 128, [5], FAKE, FAKE, [1], stream=0) == ek.ERR_NULL
    assert code(ek.window_append, sh, FAKE, FAKE, 0, 0, [5], FAKE, FAKE, [1], stream=0) == ek.ERR_SHAPE
    assert code(ek.window_append, sh, FAKE, FAKE, 4, 128, [-1], FAKE, FAKE, [1], stream=0) == ek.ERR_SHAPE
    assert code(ek.window_append, sh, FAKE, FAKE, 4, 128, [5], FAKE, FAKE, [-2], stream=0) == ek.ERR_SHAPE
    assert code(ek.window_append, sh, FAKE, FAKE, 4, 128, [5], None, FAKE, [1], stream=0) == ek.ERR_NULL
    assert code(ek.window_append, sh, FAKE, FAKE, 4, 128, [5, 6], None, None, [0, 0], stream=0) == ek.OK


def test_mlp_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "bf16")
    a, t = caches()
    big = _Ws(1 << 30)
    ok = (FAKE, FAKE, FAKE, FAKE)
    assert code(ek.decode_attn_mlp, sh, a, t, *ok, 100, ek.ACT_RELU, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    assert code(ek.decode_attn_mlp, sh, a, t, *ok, 128, 0, FAKE, FAKE, None, big, stream=0) == ek.ERR_SHAPE
    assert code(ek.decode_attn_mlp, sh, a, t, None, FAKE, FAKE, FAKE, 128, ek.ACT_SILU, FAKE, FAKE, None, big,
                stream=0) == ek.ERR_NULL
    assert code(ek.decode_attn_mlp, sh, a, t, *ok, 128, ek.ACT_RELU, FAKE, FAKE, None, _Ws(64), stream=0) == ek.ERR_WORKSPACE
    f32 = ek.make_shape(8, 8, 64, 256, "f32")
    assert code(ek.decode_attn_mlp, f32, a, t, *ok, 128, ek.ACT_RELU, FAKE, FAKE, None, big, stream=0) == ek.ERR_UNSUPPORTED
    assert ek.mlp_workspace_bytes(f32, 1, 100, 128) == 0
    assert ek.mlp_workspace_bytes(sh, 1, 100, 128) > 0
    assert ek.mlp_workspace_bytes(sh, 1, 100, 96) == 0


def test_fit_argument_errors(lib):
    sh = ek.make_shape(8, 8, 64, 256, "bf16")
    big = _Ws(1 << 34)
    assert ek.fit_workspace_bytes(sh, 4096) > 0
    assert ek.fit_workspace_bytes(sh, 100) == 0                       # rows not a multiple of 64
    assert ek.fit_workspace_bytes(ek.make_shape(8, 8, 64, 256, "f32"), 4096) == 0
    assert ek.fit_workspace_bytes(ek.make_shape(8, 8, 64, 512, "bf16"), 4096) == 0   # nothing to predict
    assert code(ek.fit_linear, sh, None, FAKE, 4096, FAKE, big, stream=0) == ek.ERR_NULL
    assert code(ek.fit_linear, sh, FAKE, FAKE, 100, FAKE, big, stream=0) == ek.ERR_SHAPE
    assert code(ek.fit_linear, sh, FAKE, FAKE, 4096, FAKE, big, ridge=-1.0, stream=0) == ek.ERR_SHAPE
    assert code(ek.fit_linear, sh, FAKE, FAKE, 4096, FAKE, big, max_iters=0, stream=0) == ek.ERR_SHAPE
    assert code(ek.fit_linear, sh, FAKE, FAKE, 4096, FAKE, _Ws(1024), stream=0) == ek.ERR_WORKSPACE
    assert code(ek.fit_linear, sh, FAKE, FAKE, 1 << 22, FAKE, big, stream=0) == ek.ERR_UNSUPPORTED   # > 2 GB per matrix
    # a narrow layer (D = 128) stays under 2 GB per matrix far longer, but the transposed input's row
    # pitch (n_rows * 2 bytes) must fit the kernel's 24-bit multiply and its 2 GB window
    narrow = ek.make_shape(2, 2, 64, 64, "bf16")
    assert ek.fit_workspace_bytes(narrow, 1 << 21) > 0
    assert ek.fit_workspace_bytes(narrow, 4177920) > 0                # 257 * n * 2 just under 2^31
    assert ek.fit_workspace_bytes(narrow, 4177920 + 128) == 0
    assert ek.fit_workspace_bytes(narrow, 1 << 23) == 0
    assert code(ek.fit_linear, narrow, FAKE, FAKE, 1 << 23, FAKE, big, stream=0) == ek.ERR_UNSUPPORTED


def test_decode_path_query(lib):
    sh = lambda *a, **k: ek.make_shape(*a, **k)
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16")) == ek.PATH_FUSED
    assert ek.decode_path(sh(32, 8, 128, 512, "bf16")) == ek.PATH_FUSED             # G = 4
    assert ek.decode_path(sh(64, 8, 128, 512, "bf16")) == ek.PATH_FUSED             # G = 8: the limit
    assert ek.decode_path(sh(128, 8, 128, 512, "bf16")) == ek.PATH_UNFUSED          # G = 16: 16 pairs > 8
    assert ek.decode_path(sh(64, 8, 64, 256, "bf16")) == ek.PATH_UNFUSED            # d = 64, G = 8: 16 pairs
    assert ek.decode_path(sh(32, 8, 64, 256, "bf16")) == ek.PATH_FUSED              # d = 64, G = 4: 8 pairs
    assert ek.decode_path(sh(8, 8, 64, 256, "f32")) == ek.PATH_FUSED
    assert ek.decode_path(sh(8, 8, 64, 512, "f32")) == ek.PATH_RETAINED_ONLY
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16", flags=ek.FLAG_UNFUSED)) == ek.PATH_UNFUSED
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16", flags=ek.FLAG_W_PACKED)) == ek.PATH_FUSED_DIRECT
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16", flags=ek.FLAG_W_PACKED | ek.FLAG_STAGED)) == ek.PATH_FUSED
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16", flags=ek.FLAG_ABSORBED)) == ek.PATH_ABSORBED
    assert ek.decode_path(sh(32, 32, 128, 2048, "bf16", flags=ek.FLAG_ABSORB_V)) == ek.PATH_ABSORB_V
    assert code(ek.decode_path, sh(128, 8, 128, 512, "bf16", flags=ek.FLAG_W_PACKED)) == ek.ERR_UNSUPPORTED
    assert code(ek.decode_path, sh(8, 8, 64, 256, "f32", flags=ek.FLAG_ABSORBED)) == ek.ERR_UNSUPPORTED
    assert code(ek.decode_path, sh(8, 8, 96, 256, "bf16")) == ek.ERR_UNSUPPORTED
    # the workspace query already covers the materialising path such a layer takes
    big, small = sh(128, 8, 128, 512, "bf16"), sh(64, 8, 128, 512, "bf16", flags=ek.FLAG_UNFUSED)
    assert ek.workspace_bytes(big, 2, 5000) >= ek.workspace_bytes(small, 2, 5000) > 5000 * 512 * 2 * 2


def test_compress_in_place_argument_rules(lib):
    sh = ek.make_shape(8, 8, 64, 256, "bf16")
    full = ek.LayerCache(FAKE, FAKE, 512, 512, [0, 256], [0, 0], [256, 256])     # no valid rows: nothing launched
    same = ek.LayerCache(FAKE, FAKE, 256, 512, [0, 256], [0, 0], [256, 256])
    assert code(ek.cache_compress, sh, full, same, stream=0) == ek.OK
    moved = ek.LayerCache(FAKE, FAKE, 256, 1024, [0, 512], [0, 0], [256, 256])
    assert code(ek.cache_compress, sh, full, moved, stream=0) == ek.ERR_UNSUPPORTED   # in place keeps the row indices
    inside = ek.LayerCache(FAKE + 4096, FAKE + 4096, 256, 512, [0, 256], [0, 0], [256, 256])
    assert code(ek.cache_compress, sh, full, inside, stream=0) == ek.ERR_UNSUPPORTED  # partial overlap
    crossed = ek.LayerCache(FAKE, FAKE + (1 << 30), 256, 512, [0, 256], [0, 0], [256, 256])
    assert code(ek.cache_compress, sh, full, crossed, stream=0) == ek.ERR_UNSUPPORTED


def test_every_status_check_in_the_binding_is_well_formed():
    """_check(status, label): a slip in an edit once gave one of these calls extra labels, which
    only shows when that wrapper runs on a GPU."""
    import ast
    tree = ast.parse(open(os.path.join(ROOT, "paper_2603_22910_amd", "binding.py")).read())
    calls = [n for n in ast.walk(tree) if isinstance(n, ast.Call) and getattr(n.func, "id", "") == "_check"]
    assert len(calls) >= 12
    for c in calls:
        assert len(c.args) == 2 and not c.keywords, ast.dump(c)[:200]
        assert isinstance(c.args[1], ast.Constant) and c.args[1].value in ek.EXPORTS
