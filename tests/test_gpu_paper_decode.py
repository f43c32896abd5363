"""GPU parity of the paper-faithful decode (rotary embedding after reconstruction,
uncompressed sink + local window) against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload, error_metrics

import oracle_ref as ref

pytestmark = pytest.mark.gpu

TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-5, 1e-5)}
MODES = [pytest.param(0, id="fused"), pytest.param(ek.FLAG_UNFUSED, id="unfused"),
         pytest.param(-1, id="packed"), pytest.param(ek.FLAG_ABSORB_V, id="absorb_v")]


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def check(got, want, dtype, what):
    mx, rl = error_metrics(got, want)
    print(f"[parity] {what}: max_abs={mx:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all(), what
    assert mx <= TOL[dtype][0] and rl <= TOL[dtype][1], f"{what}: max_abs={mx:.3e} rel_l2={rl:.3e}"


def run(w, flags, use_rope, use_window, n_sink=4, n_recent=128):
    inp = synth.generate(w)
    if flags == -1:
        if w.dtype != "bf16" or w.d_out == 0 or w.n_retained % w.head_dim:
            pytest.skip("packed weights: bf16 fused path, whole heads only")
        dw = DeviceWorkload(inp)
        dw.pack_weights()
        dw.W_K, dw.W_V = dw.W_K_packed, dw.W_V_packed
    else:
        if flags & ek.FLAG_ABSORB_V and w.dtype != "bf16":
            pytest.skip("value-absorbed decode: bf16 caches only")
        dw = DeviceWorkload(inp, flags=flags)
    rope = synth.rope_tables(w.head_dim, max(inp.seq_len[:inp.n_decode]) + 3) if use_rope else None
    window = (*synth.window_rows(inp, n_sink, n_recent), n_sink, n_recent) if use_window else None
    out, lse = dw.decode_ex(rope, window)
    torch.cuda.synchronize()
    o_ref, l_ref = ref.decode_paper_ref(inp, rope, window)
    check(host(out), o_ref, w.dtype, f"{w.name} rope={use_rope} window={use_window} flags={flags}")
    lt = 1e-5 if w.dtype == "f32" else 2e-2
    assert np.abs(host(lse) - l_ref).max() <= lt
    return inp, dw, rope, window


EXTRAS = [pytest.param(True, False, id="rope"), pytest.param(False, True, id="window"),
          pytest.param(True, True, id="rope+window")]


@pytest.mark.parametrize("use_rope,use_window", EXTRAS)
@pytest.mark.parametrize("flags", MODES)
@pytest.mark.parametrize("H_q,H_kv,d,m,dtype", [
    (8, 8, 128, 512, "bf16"),      # MHA, half retained (the 7B-shaped layout, reduced)
    (32, 8, 128, 512, "bf16"),     # GQA 4:1 (the paper's 8 x 128 layout)
    (8, 4, 64, 128, "bf16"),       # head_dim 64
    (32, 8, 128, 0, "bf16"),       # nothing retained (the paper's ratio-0.5 preset)
    (32, 8, 128, 64, "bf16"),      # half a head retained (the paper's m = 64 preset)
    (8, 8, 64, 256, "f32"),
])
def test_decode_extras_shapes(H_q, H_kv, d, m, dtype, flags, use_rope, use_window):
    w = synth.Workload(f"px_{H_q}_{H_kv}_{d}_{m}_{dtype}", dtype, H_q, H_kv, d, m, seed=300 + H_q + m,
                       seq_lens=(700, 133, 390) if dtype == "bf16" else (300, 140))
    run(w, flags, use_rope, use_window)


@pytest.mark.parametrize("flags", [pytest.param(0, id="fused"), pytest.param(ek.FLAG_ABSORB_V, id="absorb_v")])
@pytest.mark.parametrize("L", [1, 3, 4, 5, 131, 132, 133, 134, 259, 260, 261, 400, 1030])
def test_window_boundaries(L, flags):
    """Lengths around n_sink, n_sink + n_recent and the tile size: everything in the
    window, exactly one compressed token, ring wrap-around."""
    w = synth.Workload(f"pw_L{L}", "bf16", 8, 4, 128, 256, seed=500 + L, seq_lens=(L, max(1, L - 1)))
    run(w, flags, True, True)


@pytest.mark.parametrize("flags", [pytest.param(0, id="fused"), pytest.param(ek.FLAG_ABSORB_V, id="absorb_v")])
@pytest.mark.parametrize("n_sink,n_recent", [(0, 64), (4, 0), (1, 1), (16, 200)])
def test_window_sizes(n_sink, n_recent, flags):
    w = synth.Workload(f"pw_{n_sink}_{n_recent}", "bf16", 8, 4, 128, 256, seed=41, seq_lens=(500, 17, 230))
    run(w, flags, False, True, n_sink, n_recent)


def test_extras_null_equals_plain_decode():
    w = synth.Workload("px_null", "bf16", 8, 4, 128, 256, seed=8, seq_lens=(300, 129))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    o0 = host(dw.decode()[0]).copy(); torch.cuda.synchronize()
    o1 = host(dw.decode_ex(None, None)[0]); torch.cuda.synchronize()
    assert np.array_equal(o0, o1)


def test_window_when_everything_is_in_it_ignores_the_predictor():
    """L <= n_sink + n_recent: the output depends on the window rows only."""
    w = synth.Workload("px_allwin", "bf16", 8, 4, 128, 256, seed=9, seq_lens=(100, 132))
    inp = synth.generate(w)
    window = (*synth.window_rows(inp, 4, 128), 4, 128)
    dw = DeviceWorkload(inp)
    o0 = host(dw.decode_ex(None, window)[0]).copy(); torch.cuda.synchronize()
    dw.W_K.mul_(-3.0); dw.W_V.zero_()
    o1 = host(dw.decode_ex(None, window)[0]); torch.cuda.synchronize()
    assert np.array_equal(o0, o1)


def test_window_append_keeps_the_ring_current():
    """Tokens appended in pieces through the ABI give, bit for bit, the window that
    the input generator lays out for the final lengths."""
    w = synth.Workload("px_app", "bf16", 4, 2, 128, 128, seed=13, seq_lens=(300, 7, 140))
    inp = synth.generate(w)
    n_sink, n_recent = 4, 128
    dev = torch.device("cuda:0")
    B, D = inp.n_decode, w.D
    rows = n_sink + n_recent
    # the target's full rows, token by token: retained dims from the cache, the rest seeded per token
    g = torch.Generator().manual_seed(99)
    full_k = [torch.randn(L, D, generator=g).to(w.torch_dtype) for L in inp.seq_len[:B]]
    full_v = [torch.randn(L, D, generator=g).to(w.torch_dtype) for L in inp.seq_len[:B]]
    win_k = torch.zeros(B, rows, D, dtype=w.torch_dtype, device=dev)
    win_v = torch.zeros_like(win_k)
    sh = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_retained, w.dtype)
    have = [0] * B
    rng = np.random.default_rng(3)
    while any(h < L for h, L in zip(have, inp.seq_len[:B])):
        n_new = [int(min(L - h, rng.integers(0, 200))) for h, L in zip(have, inp.seq_len[:B])]
        kn = torch.cat([full_k[b][have[b]:have[b] + n_new[b]] for b in range(B)]).to(dev)
        vn = torch.cat([full_v[b][have[b]:have[b] + n_new[b]] for b in range(B)]).to(dev)
        ek.window_append(sh, win_k, win_v, n_sink, n_recent, have, kn, vn, n_new)
        have = [h + n for h, n in zip(have, n_new)]
    torch.cuda.synchronize()
    wk, wv = win_k.cpu(), win_v.cpu()
    for b, L in enumerate(inp.seq_len[:B]):
        for p in range(L):
            if p < n_sink or p >= L - n_recent:
                r = p if p < n_sink else n_sink + (p - n_sink) % n_recent
                assert torch.equal(wk[b, r], full_k[b][p]), (b, p)
                assert torch.equal(wv[b, r], full_v[b][p]), (b, p)


@pytest.mark.parametrize("flags", [pytest.param(0, id="fused"), pytest.param(ek.FLAG_ABSORB_V, id="absorb_v")])
def test_decode_extras_batch_above_one_launch(flags):
    lens = tuple(1 + (53 * i) % 400 for i in range(140))
    w = synth.Workload("px_b140", "bf16", 4, 2, 128, 128, seed=78, seq_lens=lens)
    run(w, flags, True, True)


def test_decode_extras_full_size_sampled():
    """The paper's GQA layout at 32 K tokens (8 x 128 KV heads, half retained) with both
    extras; sampled heads against the oracle."""
    from oracle import echokv_oracle as orc
    w = synth.CONFIGS[3].scaled(seq_lens=(32768,))
    inp = synth.generate(w)
    rope = synth.rope_tables(w.head_dim, 32768)
    window = (*synth.window_rows(inp, 4, 128), 4, 128)
    dw = DeviceWorkload(inp, flags=ek.FLAG_ABSORB_V)       # workspace sized for both paths
    o_ref, l_ref = ref.decode_paper_ref(inp, rope, window)
    for name, fl in (("fused", 0), ("absorb_v", ek.FLAG_ABSORB_V)):
        dw.set_flags(fl)
        out, lse = dw.decode_ex(rope, window); torch.cuda.synchronize()
        got = host(out)
        assert np.isfinite(got).all()
        check(got, o_ref, "bf16", f"cfg3-shaped 32K rope+window, {name}")
        assert np.abs(host(lse) - l_ref).max() <= 2e-2


# ---- causal prefill with the rotary embedding ---------------------------------------
@pytest.mark.parametrize("H_q,H_kv,d,m,dtype,plen,pq", [
    (8, 8, 128, 512, "bf16", 400, 300),       # short-chunk kernel, MHA, half retained
    (8, 2, 128, 128, "bf16", 1400, 1090),     # long-chunk kernel, GQA 4:1, ragged
    (8, 4, 64, 128, "bf16", 1200, 1200),      # head_dim 64, whole sequence in one chunk
    (32, 8, 128, 0, "bf16", 300, 64),         # nothing retained
    (4, 4, 128, 512, "bf16", 260, 200),       # everything retained
    (32, 8, 128, 64, "bf16", 330, 300),       # half a head retained (the paper's m = 64 preset)
    (8, 8, 64, 256, "f32", 200, 150),         # fp32: the streaming path rotates in the kernel
    (8, 2, 128, 128, "bf16", 4300, 333),      # short chunk in front of a long context: keys cut into shares
    (32, 8, 128, 64, "bf16", 2100, 130),      # the same with the paper's m = 64 preset
])
def test_prefill_rope(H_q, H_kv, d, m, dtype, plen, pq):
    w = synth.Workload(f"ppx_{H_q}_{H_kv}_{d}_{m}_{dtype}", dtype, H_q, H_kv, d, m, seed=700 + H_q + m,
                       seq_lens=(5,), prefill_len=plen, prefill_q=pq)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    rope = synth.rope_tables(d, plen + 2)
    out, lse = dw.prefill_ex(rope)
    torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_paper_ref(inp, rope)
    check(host(out), o_ref, dtype, f"{w.name} prefill rope")
    assert np.abs(host(lse) - l_ref).max() <= (1e-5 if dtype == "f32" else 2e-2)
    # without tables the _ex entry point is the plain prefill, bit for bit
    got = host(out).copy()
    o0, _ = dw.prefill(); torch.cuda.synchronize()
    plain = host(o0).copy()
    ek.prefill_attn_ex(dw.shape, dw.anchor_all, dw.target_all, dw.W_K, dw.W_V, inp.n_decode, dw.q_prefill,
                       pq, inp.q_pos0, dw.out_prefill, dw.lse_prefill, dw.workspace)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(dw.out_prefill), plain)
    assert np.abs(got - plain).max() > 1e-3          # and the rotation does change the result


def test_prefill_rope_last_row_equals_decode_ex():
    """The chunk's last query against the decode entry point with the same tables."""
    w = synth.Workload("ppx_last", "bf16", 8, 4, 128, 256, seed=731, seq_lens=(5,), prefill_len=300, prefill_q=40)
    inp = synth.generate(w)
    rope = synth.rope_tables(128, 310)
    dw = DeviceWorkload(inp, out_dtype="f32")
    out, _ = dw.prefill_ex(rope); torch.cuda.synchronize()
    b = inp.n_decode
    single = synth.Inputs(w, [inp.seq_start[b]], [inp.seq_len[b]], [inp.seq_cap[b]], 1, inp.K_a, inp.V_a,
                          inp.K_r, inp.V_r, inp.W_K, inp.W_V, inp.q_prefill[-1:].clone(), None, 0)
    dd = DeviceWorkload(single, out_dtype="f32")
    o_dec, _ = dd.decode_ex(rope, None); torch.cuda.synchronize()
    np.testing.assert_allclose(host(out)[-1], host(o_dec)[0], rtol=2e-2, atol=6e-3)   # bf16 K_hat, rotated keys rounded
