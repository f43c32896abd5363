"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on
the same seeded inputs.  Tolerances are the benchmark's: bf16 inputs max-abs
<= 2e-2 and relative L2 <= 5e-3; fp32 inputs <= 1e-5 for both."""
import math

import numpy as np
import pytest
import torch

from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload, error_metrics

import oracle_ref as ref

pytestmark = pytest.mark.gpu

TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-5, 1e-5)}
PACKED = 1 << 20       # test-only marker: weights re-laid out once by echokv_pack_weights (direct-to-LDS kernel)
MODES = [pytest.param(0, id="fused"), pytest.param(ek.FLAG_UNFUSED, id="unfused"),
         pytest.param(PACKED, id="packed"),
         pytest.param(PACKED | ek.FLAG_STAGED, id="packed_staged"),
         pytest.param(ek.FLAG_ABSORBED, id="absorbed"),
         pytest.param(ek.FLAG_ABSORB_V, id="absorb_v")]


def check(got, want, dtype, what=""):
    mx, rl = error_metrics(got, want)
    tmx, trl = TOL[dtype]
    print(f"[parity] {what}: max_abs={mx:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(got).all(), what
    assert mx <= tmx and rl <= trl, f"{what}: max_abs={mx:.3e} rel_l2={rl:.3e}"


def host(t):
    return t.float().cpu().double().numpy()


def make_dw(inp, flags, **kw):
    if flags & PACKED:
        w = inp.w
        if w.dtype != "bf16" or w.d_out == 0:
            pytest.skip("packed weights: bf16 fused path with something to predict only")
        dw = DeviceWorkload(inp, flags=0, **kw)
        dw.pack_weights()
        dw.shape.flags |= flags & ek.FLAG_STAGED
        return dw
    if flags & (ek.FLAG_ABSORBED | ek.FLAG_ABSORB_V) and inp.w.dtype != "bf16":
        pytest.skip("weight-absorbed decode: bf16 caches only")
    return DeviceWorkload(inp, flags=flags, **kw)


def run_decode_case(w, flags, out_dtype=None, lse_tol=None):
    inp = synth.generate(w)
    dw = make_dw(inp, flags, out_dtype=out_dtype)
    out, lse = dw.decode()
    torch.cuda.synchronize()
    o_ref, l_ref = ref.decode_ref(inp)
    check(host(out), o_ref, w.dtype, f"{w.name} decode flags={flags}")
    lt = lse_tol or (1e-5 if w.dtype == "f32" else 2e-2)
    assert np.abs(host(lse) - l_ref).max() <= lt
    return inp, dw


# ---- reduced-size versions of the five configurations (every element checked) ----
SMALL = {
    0: synth.CONFIGS[0],                                            # full size already
    1: synth.CONFIGS[1].scaled(seq_lens=(700, 513, 256, 1)),
    2: synth.CONFIGS[2].scaled(seq_lens=(1111, 384)),
    3: synth.CONFIGS[3].scaled(seq_lens=(2500,)),
    4: synth.CONFIGS[4].scaled(batch=6, len_lo=16, len_hi=1500, prefill_len=400, prefill_q=400),
}


@pytest.mark.parametrize("flags", MODES)
@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4])
def test_decode_small(cfg, flags):
    run_decode_case(SMALL[cfg], flags)


@pytest.mark.parametrize("flags", MODES)
def test_decode_f32_output_from_bf16_cache(flags):
    run_decode_case(SMALL[1].scaled(seq_lens=(300, 129)), flags, out_dtype="f32")


@pytest.mark.parametrize("flags", MODES)
@pytest.mark.parametrize("L", [1, 2, 63, 64, 127, 128, 129, 255, 256, 257, 511, 513])
def test_decode_tile_boundaries(L, flags):
    w = synth.Workload(f"edge_L{L}", "bf16", 8, 4, 128, 256, seed=100 + L, seq_lens=(L, max(1, L - 1)))
    run_decode_case(w, flags)


@pytest.mark.parametrize("flags", MODES)
@pytest.mark.parametrize("H_q,H_kv,d,m,dtype", [
    (4, 4, 128, 0, "bf16"),        # nothing retained: anchor-only predictor input
    (4, 4, 128, 512, "bf16"),      # everything retained: ordinary attention
    (8, 4, 64, 128, "bf16"),       # head_dim 64, G = 2
    (16, 2, 128, 128, "bf16"),     # G = 8
    (3, 3, 128, 128, "bf16"),      # d_out = 256 not filling a 256-wide tile evenly with 3 heads
    (6, 3, 128, 128, "bf16"),
    (5, 5, 128, 128, "bf16"),      # 4 predicted heads + odd retained count
    (1, 1, 64, 0, "bf16"),         # one k-tile only (d_in = 64), one predicted head
    (2, 2, 64, 64, "bf16"),        # three k-tiles (odd tail)
    (2, 1, 128, 0, "bf16"),        # two k-tiles, G = 2
    (1, 1, 64, 0, "f32"),
    (4, 2, 128, 128, "f32"),
    (8, 8, 64, 0, "f32"),
    (8, 4, 64, 256, "f32"),        # full retention fp32
])
def test_decode_shapes(H_q, H_kv, d, m, dtype, flags):
    w = synth.Workload(f"shape_{H_q}_{H_kv}_{d}_{m}_{dtype}", dtype, H_q, H_kv, d, m, seed=7,
                       seq_lens=(333, 64, 130))
    run_decode_case(w, flags)


def test_pack_weights_is_a_transpose_and_flag_is_checked():
    w = SMALL[1].scaled(seq_lens=(100,))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    dw.pack_weights(); torch.cuda.synchronize()
    assert torch.equal(dw.W_K_packed.cpu(), inp.W_K.t().contiguous())
    assert torch.equal(dw.W_V_packed.cpu(), inp.W_V.t().contiguous())
    with pytest.raises(ek.EchoKVError) as e:          # packed layout only feeds the fused decode
        ek.reconstruct(dw.shape, dw.anchor_all, dw.target_all, dw.W_K_packed, dw.W_V_packed, 0, 0, 10,
                       dw.out, dw.out)
    assert e.value.code == ek.ERR_UNSUPPORTED
    dw.shape.flags |= ek.FLAG_UNFUSED
    with pytest.raises(ek.EchoKVError) as e:
        dw.decode()
    assert e.value.code == ek.ERR_UNSUPPORTED


def test_decode_custom_scale():
    w = SMALL[1].scaled(seq_lens=(300,))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, softmax_scale=0.05)
    out, _ = dw.decode(); torch.cuda.synchronize()
    o_ref, _ = ref.decode_ref(inp, scale=0.05)
    check(host(out), o_ref, "bf16", "custom scale")


@pytest.mark.parametrize("flags", MODES)
def test_decode_is_deterministic(flags):
    inp = synth.generate(SMALL[4])
    dw = make_dw(inp, flags)
    a = dw.decode()[0].clone(); b = dw.decode()[0].clone()
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("flags", MODES)
def test_selector_weights_copy_heads_exactly(flags):
    """W that copies anchor head columns: predicted heads equal stored anchor
    heads bit for bit (1*x + zeros in fp32, re-rounding a bf16 value is exact)."""
    w = synth.Workload("selector", "bf16", 4, 4, 128, 256, seed=11, seq_lens=(300,))
    inp = synth.generate(w)
    src = list(range(128, 256)) + [w.D + i for i in range(128)]     # anchor head 1, retained head 0
    inp.W_K = synth.selector_weights(w, src); inp.W_V = synth.selector_weights(w, src)
    dw = DeviceWorkload(inp, flags=0 if flags & PACKED else flags)
    k_out, v_out = dw.reconstruct(0, 0, 300); torch.cuda.synchronize()
    if flags & PACKED:
        dw.pack_weights()
        dw.shape.flags |= flags & ek.FLAG_STAGED
    X = torch.cat([inp.K_a[:300], inp.K_r[:300]], dim=1)
    assert torch.equal(k_out.cpu()[:, :256], inp.K_r[:300])
    assert torch.equal(k_out.cpu()[:, 256:], X[:, src])
    out, _ = dw.decode(); torch.cuda.synchronize()
    o_ref, _ = ref.decode_ref(inp)
    check(host(out), o_ref, "bf16", "selector decode")
    # heads 2 and 3 see copies of anchor head 1 / retained head 0: head 3 == head 0 given equal q
    inp.q[0, 3] = inp.q[0, 0]
    dw2 = make_dw(inp, flags, out_dtype="f32")
    o2 = host(dw2.decode()[0]); torch.cuda.synchronize()
    o2 = host(dw2.out)
    np.testing.assert_allclose(o2[0, 3], o2[0, 0], rtol=2e-5, atol=2e-6)


@pytest.mark.parametrize("cfg", [0, 1, 3])
def test_reconstruct_small(cfg):
    w = SMALL[cfg]
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    L = inp.seq_len[0]
    t0, t1 = (3, L - 2) if L > 8 else (0, L)
    k_out, v_out = dw.reconstruct(0, t0, t1); torch.cuda.synchronize()
    k_ref, v_ref = ref.reconstruct_ref(inp, 0, t0, t1)
    # retained part is a copy: exact
    assert np.array_equal(host(k_out)[:, :w.n_retained], k_ref[:, :w.n_retained])
    tol = (1e-5, 1e-5) if w.dtype == "f32" else (2e-2, 5e-3)
    for got, want, nm in ((k_out, k_ref, "K"), (v_out, v_ref, "V")):
        mx, rl = error_metrics(host(got), want)
        print(f"[parity] {w.name} reconstruct {nm}: max_abs={mx:.3e} rel_l2={rl:.3e}")
        assert mx <= tol[0] and rl <= tol[1]


def test_cache_append_matches_the_oracle_layout():
    """Tokens appended in pieces through the ABI against the oracle's cache_append fed the same
    full-width rows (Eq. 1 for the anchor, Eq. 2 for the target): bit for bit the same cache; the
    dropped dims (marker values here) are never written anywhere."""
    from oracle import echokv_oracle as orc
    w = synth.Workload("append", "bf16", 8, 8, 128, 512, seed=21, seq_lens=(200, 77, 300))
    inp = synth.generate(w)
    dev = torch.device("cuda:0")
    shape = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_retained, "bf16")
    pool = inp.pool_tokens
    Ka = torch.zeros(pool, w.D, dtype=torch.bfloat16, device=dev); Va = torch.zeros_like(Ka)
    Kr = torch.zeros(pool, w.n_retained, dtype=torch.bfloat16, device=dev); Vr = torch.zeros_like(Kr)
    zero = [0] * 3
    anchor = ek.LayerCache(Ka, Va, w.D, pool, inp.seq_start, zero, inp.seq_cap)
    target = ek.LayerCache(Kr, Vr, w.n_retained, pool, inp.seq_start, zero, inp.seq_cap)
    # the oracle's caches (fp64 holds every bf16 value exactly) and its own sequence lengths
    o_Ka = np.zeros((pool, w.D)); o_Va = np.zeros((pool, w.D))
    o_Kr = np.zeros((pool, w.n_retained)); o_Vr = np.zeros((pool, w.n_retained))
    o_len_a = [0, 0, 0]; o_len_t = [0, 0, 0]
    # the target layer's full K/V rows: retained dims as generated, dropped dims = a marker
    done = [0, 0, 0]
    steps = [[150, 77, 1], [50, 0, 299]]
    for n_new in steps:
        ka, va, kt, vt = [], [], [], []
        for b, n in enumerate(n_new):
            r = slice(inp.seq_start[b] + done[b], inp.seq_start[b] + done[b] + n)
            ka.append(inp.K_a[r]); va.append(inp.V_a[r])
            full_k = torch.full((n, w.D), 77.0, dtype=torch.bfloat16); full_k[:, :w.n_retained] = inp.K_r[r]
            full_v = torch.full((n, w.D), -77.0, dtype=torch.bfloat16); full_v[:, :w.n_retained] = inp.V_r[r]
            kt.append(full_k); vt.append(full_v)
            done[b] += n
            orc.cache_append(o_Ka, inp.seq_start[b], o_len_a[b], ref.f64(ka[-1]))
            o_len_a[b] = orc.cache_append(o_Va, inp.seq_start[b], o_len_a[b], ref.f64(va[-1]))
            orc.cache_append(o_Kr, inp.seq_start[b], o_len_t[b], ref.f64(full_k))
            o_len_t[b] = orc.cache_append(o_Vr, inp.seq_start[b], o_len_t[b], ref.f64(full_v))
        cat = lambda xs: torch.cat(xs).to(dev)
        ek.cache_append(shape, anchor, cat(ka), cat(va), n_new)
        ek.cache_append(shape, target, cat(kt), cat(vt), n_new)
    torch.cuda.synchronize()
    assert list(anchor.seq_len) == o_len_a and list(target.seq_len) == o_len_t == inp.seq_len
    for got, want in ((Ka, o_Ka), (Va, o_Va), (Kr, o_Kr), (Vr, o_Vr)):
        assert np.array_equal(host(got), want)
    assert not (np.abs(host(Kr)) == 77.0).any() and not (np.abs(host(Vr)) == 77.0).any()
    # and the generator's bulk layout is the same cache
    assert torch.equal(Ka.cpu(), inp.K_a) and torch.equal(Kr.cpu(), inp.K_r)
    with pytest.raises(ek.EchoKVError) as e:
        ek.cache_append(shape, target, Ka, Va, [1000, 0, 0])
    assert e.value.code == ek.ERR_CAPACITY


@pytest.mark.parametrize("flags", MODES)
def test_decode_growing_scores(flags):
    """Key rows whose norm grows fourfold along the sequence: the score maxima of successive
    tiles and splits differ by many powers of two, so every rescale and the split merge are
    exercised with large exponents."""
    w = synth.Workload("dec_grow", "bf16", 8, 4, 128, 256, seed=39, seq_lens=(1500, 700))
    inp = synth.generate(w)
    for b in range(inp.n_decode):
        r = inp.rows(b)
        L = inp.seq_len[b]
        ramp = (1.0 + 3.0 * torch.arange(L, dtype=torch.float32) / L)[:, None]
        inp.K_a[r] = (inp.K_a[r].float() * ramp).to(inp.K_a.dtype)
        inp.K_r[r] = (inp.K_r[r].float() * ramp).to(inp.K_r.dtype)
    dw = make_dw(inp, flags)
    out, lse = dw.decode(); torch.cuda.synchronize()
    o_ref, l_ref = ref.decode_ref(inp)
    check(host(out), o_ref, w.dtype, f"decode, growing scores, flags={flags}")
    assert np.abs(host(lse) - l_ref).max() <= 5e-2      # scores reach +-30: bf16 inputs, fp32 sums


# ---- prefill -------------------------------------------------------------------
def run_prefill_case(w, flags=0):
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, flags=flags)
    out, lse = dw.prefill(); torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_ref(inp)
    check(host(out), o_ref, w.dtype, f"{w.name} prefill")
    assert np.abs(host(lse) - l_ref).max() <= (1e-5 if w.dtype == "f32" else 2e-2)
    return inp, dw


# chunks of 1024 queries and more take the kernel variant with 64 queries per wave
@pytest.mark.parametrize("plen,pq", [(400, 400), (400, 150), (130, 1), (257, 256), (64, 64),
                                     (1300, 1100), (1024, 1024), (1500, 1025)])
def test_prefill_small(plen, pq):
    run_prefill_case(SMALL[4].scaled(prefill_len=plen, prefill_q=pq))


def test_prefill_gqa_and_f32():
    run_prefill_case(synth.Workload("pf_gqa", "bf16", 8, 2, 128, 128, seed=31, seq_lens=(5,),
                                    prefill_len=300, prefill_q=200))
    run_prefill_case(synth.Workload("pf_f32", "f32", 8, 8, 64, 256, seed=32, seq_lens=(5,),
                                    prefill_len=200, prefill_q=200))
    run_prefill_case(synth.Workload("pf_full", "bf16", 4, 4, 128, 512, seed=33, seq_lens=(5,),
                                    prefill_len=200, prefill_q=100))
    run_prefill_case(synth.Workload("pf_none", "bf16", 4, 4, 128, 0, seed=34, seq_lens=(5,),
                                    prefill_len=200, prefill_q=100))
    run_prefill_case(synth.Workload("pf_gqa_long", "bf16", 8, 2, 128, 128, seed=35, seq_lens=(5,),
                                    prefill_len=1400, prefill_q=1090))
    run_prefill_case(synth.Workload("pf_d64_long", "bf16", 4, 4, 64, 128, seed=36, seq_lens=(5,),
                                    prefill_len=1200, prefill_q=1200))


# a short chunk in front of a long context: the long-chunk kernel with the keys of every (head, query
# block) cut into shares (one workgroup each) and a merge of the shares' partial softmax sums
@pytest.mark.parametrize("plen,pq", [(1400, 300), (3000, 500), (5000, 1000), (2049, 1), (2049, 2), (4100, 385),
                                     (8200, 100), (1024, 1023), (1100, 769)])
def test_prefill_short_chunk_long_context(plen, pq):
    w = SMALL[4].scaled(prefill_len=plen, prefill_q=pq)
    assert ek.workspace_bytes(ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_retained, "bf16"), 1, plen, pq) > 0
    run_prefill_case(w)


def test_prefill_short_chunk_long_context_shapes():
    run_prefill_case(synth.Workload("pfs_gqa", "bf16", 8, 2, 128, 128, seed=131, seq_lens=(5,),
                                    prefill_len=4200, prefill_q=200))          # 8 shares
    run_prefill_case(synth.Workload("pfs_d64", "bf16", 4, 4, 64, 128, seed=132, seq_lens=(5,),
                                    prefill_len=3000, prefill_q=700))
    run_prefill_case(synth.Workload("pfs_none", "bf16", 4, 4, 128, 0, seed=133, seq_lens=(5,),
                                    prefill_len=2500, prefill_q=390))
    run_prefill_case(synth.Workload("pfs_full", "bf16", 4, 4, 128, 512, seed=134, seq_lens=(5,),
                                    prefill_len=2500, prefill_q=64))
    inp = synth.generate(synth.Workload("pfs_f32out", "bf16", 8, 4, 128, 256, seed=135, seq_lens=(5,),
                                        prefill_len=3111, prefill_q=600))
    dw = DeviceWorkload(inp, out_dtype="f32")
    out, lse = dw.prefill(); torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_ref(inp)
    check(host(out), o_ref, "bf16", "prefill short chunk, long context, f32 out")
    assert np.abs(host(lse) - l_ref).max() <= 2e-2


def test_prefill_short_chunk_long_context_growing_scores():
    """Shares that start on or next to the diagonal (queries with no visible key yet in a share) and
    maxima that keep moving inside every share."""
    w = synth.Workload("pfs_grow", "bf16", 4, 4, 128, 512, seed=137, seq_lens=(5,),
                       prefill_len=3000, prefill_q=900)
    inp = synth.generate(w)
    r = inp.rows(inp.n_decode)
    L = inp.seq_len[inp.n_decode]
    ramp = (1.0 + 10.0 * torch.arange(L, dtype=torch.float32) / L)[:, None]
    inp.K_r[r] = (inp.K_r[r].float() * ramp).to(inp.K_r.dtype)
    dw = DeviceWorkload(inp)
    out, lse = dw.prefill(); torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_ref(inp)
    check(host(out), o_ref, w.dtype, "prefill short chunk, growing scores")
    assert np.abs(host(lse) - l_ref).max() <= 2e-2


def test_prefill_growing_scores():
    """Keys whose norm grows along the sequence: the running maxima keep moving, so the
    long-chunk kernel has to raise its reference maxima and rescale several times."""
    w = synth.Workload("pf_grow", "bf16", 4, 4, 128, 512, seed=37, seq_lens=(5,),
                       prefill_len=1300, prefill_q=1200)
    inp = synth.generate(w)
    r = inp.rows(inp.n_decode)
    L = inp.seq_len[inp.n_decode]
    ramp = (1.0 + 10.0 * torch.arange(L, dtype=torch.float32) / L)[:, None]
    inp.K_r[r] = (inp.K_r[r].float() * ramp).to(inp.K_r.dtype)
    dw = DeviceWorkload(inp)
    out, lse = dw.prefill(); torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_ref(inp)
    check(host(out), o_ref, w.dtype, "prefill, growing scores")
    assert np.abs(host(lse) - l_ref).max() <= 2e-2


def test_prefill_long_chunk_f32_out():
    """fp32 outputs of the long-chunk kernel (no output rounding: what is left is the bf16
    rounding of P and of the predicted K, V)."""
    w = synth.Workload("pf_f32out", "bf16", 8, 4, 128, 256, seed=38, seq_lens=(5,),
                       prefill_len=1411, prefill_q=1100)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, out_dtype="f32")
    out, lse = dw.prefill(); torch.cuda.synchronize()
    o_ref, l_ref = ref.prefill_ref(inp)
    check(host(out), o_ref, "bf16", "prefill long chunk, f32 out")
    assert np.abs(host(lse) - l_ref).max() <= 2e-2


def test_prefill_last_row_equals_decode():
    w = SMALL[4].scaled(prefill_len=300, prefill_q=40)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, out_dtype="f32")
    out, _ = dw.prefill(); torch.cuda.synchronize()
    # decode over the prefill sequence with its last query
    inp2 = synth.generate(w)
    b = inp.n_decode
    inp2.q = inp.q_prefill[-1:].clone()
    single = synth.Inputs(w, [inp.seq_start[b]], [inp.seq_len[b]], [inp.seq_cap[b]], 1, inp.K_a,
                          inp.V_a, inp.K_r, inp.V_r, inp.W_K, inp.W_V, inp2.q, None, 0)
    dd = DeviceWorkload(single, out_dtype="f32")
    o_dec, _ = dd.decode(); torch.cuda.synchronize()
    np.testing.assert_allclose(host(out)[-1], host(o_dec)[0], rtol=1e-2, atol=4e-3)  # bf16 K_hat in prefill


@pytest.mark.parametrize("flags", MODES)
def test_decode_more_sequences_than_one_launch_describes(flags):
    """The kernels describe at most 128 sequences per launch; larger batches
    are processed in groups."""
    lens = tuple(1 + (37 * i) % 300 for i in range(150))
    w = synth.Workload("b150", "bf16", 4, 2, 128, 128, seed=77, seq_lens=lens)
    run_decode_case(w, flags)


def test_workspace_exactly_as_reported_is_enough_and_less_is_rejected():
    w = SMALL[1]
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    need = ek.workspace_bytes(dw.shape, inp.n_decode, inp.total_decode_tokens, 0)
    assert dw.workspace.numel() == need
    out, _ = dw.decode(); torch.cuda.synchronize()
    o_ref, _ = ref.decode_ref(inp)
    check(host(out), o_ref, "bf16", "exact workspace")
    dw.workspace = dw.workspace[:4096]
    with pytest.raises(ek.EchoKVError) as e:
        dw.decode()
    assert e.value.code == ek.ERR_WORKSPACE


def test_switch_from_full_cache_to_compressed_cache():
    """On-demand transition: a target layer first served from its full cache
    (m = D, ordinary attention), then compressed in place of a rebuild."""
    from oracle import echokv_oracle as orc
    w = synth.Workload("switch", "bf16", 8, 8, 128, 512, seed=41, seq_lens=(333, 70))
    inp = synth.generate(w)
    dev = torch.device("cuda:0")
    # the target layer's full K/V: retained prefix as generated + arbitrary other dims
    g = torch.Generator().manual_seed(1)
    full_k = torch.randn(inp.pool_tokens, w.D, generator=g).to(torch.bfloat16)
    full_v = torch.randn(inp.pool_tokens, w.D, generator=g).to(torch.bfloat16)
    full_k[:, :w.n_retained] = inp.K_r; full_v[:, :w.n_retained] = inp.V_r
    shape = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_retained, "bf16")
    fk, fv = full_k.to(dev), full_v.to(dev)
    full = ek.LayerCache(fk, fv, w.D, inp.pool_tokens, inp.seq_start, inp.seq_len, inp.seq_cap)
    # compressed cache laid out differently (tight capacities) on purpose
    caps = [384, 128]; starts = [128, 0]
    ck = torch.zeros(512, w.n_retained, dtype=torch.bfloat16, device=dev); cv = torch.zeros_like(ck)
    dst = ek.LayerCache(ck, cv, w.n_retained, 512, starts, [0, 0], caps)
    ek.cache_compress(shape, full, dst); torch.cuda.synchronize()
    assert list(dst.seq_len) == inp.seq_len
    for b in range(2):
        want = orc.cache_compress(ref.f64(full_k[inp.rows(b)]), w.n_retained)
        got = ck[starts[b]:starts[b] + inp.seq_len[b]].float().cpu().double().numpy()
        assert np.array_equal(got, want)
    small = ek.LayerCache(ck, cv, w.n_retained, 512, starts, [0, 0], [384, 64])
    with pytest.raises(ek.EchoKVError) as e:
        ek.cache_compress(shape, full, small)
    assert e.value.code == ek.ERR_CAPACITY


@pytest.mark.parametrize("m,lens", [(512, (333, 70, 1)), (256, (2500,)), (960, (700, 129)), (64, (1200, 5)),
                                    (0, (100,)), (1024, (100, 30))])
def test_switch_in_place_then_decode(m, lens):
    """The same transition with no second buffer (the moment it is needed there is no memory for
    one): the pool [rows, D] is narrowed to [rows, m] where it lies.  The result must be the
    oracle's compressed cache bit for bit, and decoding from it must match the oracle."""
    from oracle import echokv_oracle as orc
    w = synth.Workload(f"switch_inplace_m{m}", "bf16", 8, 8, 128, m, seed=43, seq_lens=lens)
    inp = synth.generate(w)
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(2)
    pool = inp.pool_tokens
    full_k = torch.randn(pool, w.D, generator=g).to(torch.bfloat16)
    full_v = torch.randn(pool, w.D, generator=g).to(torch.bfloat16)
    full_k[:, :m] = inp.K_r; full_v[:, :m] = inp.V_r
    fk, fv = full_k.to(dev), full_v.to(dev)
    shape = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, m, "bf16")
    full = ek.LayerCache(fk, fv, w.D, pool, inp.seq_start, inp.seq_len, inp.seq_cap)
    # the same memory seen as [pool, m]
    ck = fk.view(-1)[:pool * m].view(pool, m) if m else None
    cv = fv.view(-1)[:pool * m].view(pool, m) if m else None
    if m:
        assert ck.data_ptr() == fk.data_ptr()
    dst = ek.LayerCache(ck if m else None, cv if m else None, m, pool, inp.seq_start, [0] * len(lens), inp.seq_cap)
    if m == 0:
        dst.k = dst.v = None
    ek.cache_compress(shape, full, dst); torch.cuda.synchronize()
    assert list(dst.seq_len) == inp.seq_len
    for b in range(inp.n_decode):
        want_k = orc.cache_compress(ref.f64(full_k[inp.rows(b)]), m)
        want_v = orc.cache_compress(ref.f64(full_v[inp.rows(b)]), m)
        if m:
            assert np.array_equal(host(ck[inp.rows(b)]), want_k)
            assert np.array_equal(host(cv[inp.rows(b)]), want_v)
    # decode from the narrowed pool
    dw = DeviceWorkload(inp)
    if m:
        dw.target = ek.LayerCache(ck, cv, m, pool, inp.seq_start, inp.seq_len, inp.seq_cap)
    out, _ = dw.decode(); torch.cuda.synchronize()
    o_ref, _ = ref.decode_ref(inp)
    check(host(out), o_ref, "bf16", f"decode after in-place switch, m={m}")


def test_switch_in_place_long_pool():
    """Enough rows for the plain-copy phase (row ranges whose destination ends below their source)
    to take over from the ordered single-workgroup phase, at a ratio close to 1 and at 1/2."""
    from oracle import echokv_oracle as orc
    dev = torch.device("cuda:0")
    for H, d, m, rows in ((8, 128, 960, 9000), (8, 128, 512, 70000), (4, 64, 64, 3000)):
        D = H * d
        g = torch.Generator().manual_seed(rows)
        full_k = torch.randn(rows, D, generator=g).to(torch.bfloat16)
        full_v = torch.randn(rows, D, generator=g).to(torch.bfloat16)
        fk, fv = full_k.to(dev), full_v.to(dev)
        shape = ek.make_shape(H, H, d, m, "bf16")
        starts, lens, caps = [0, rows // 2], [rows // 2 - 7, rows - rows // 2], [rows // 2, rows - rows // 2]
        full = ek.LayerCache(fk, fv, D, rows, starts, lens, caps)
        ck = fk.view(-1)[:rows * m].view(rows, m); cv = fv.view(-1)[:rows * m].view(rows, m)
        dst = ek.LayerCache(ck, cv, m, rows, starts, [0, 0], caps)
        ek.cache_compress(shape, full, dst); torch.cuda.synchronize()
        for b in range(2):
            r = slice(starts[b], starts[b] + lens[b])
            assert np.array_equal(host(ck[r]), orc.cache_compress(ref.f64(full_k[r]), m)), (m, rows, b)
            assert np.array_equal(host(cv[r]), orc.cache_compress(ref.f64(full_v[r]), m)), (m, rows, b)


@pytest.mark.parametrize("H_q,H_kv,d,m", [(64, 4, 128, 256), (32, 4, 64, 128)])
def test_decode_more_query_heads_per_kv_head_than_the_fused_kernel_holds(H_q, H_kv, d, m):
    """(128 / d) * G > 8: the library serves the layer on the materialising path and says so."""
    w = synth.Workload(f"g{H_q // H_kv}_d{d}", "bf16", H_q, H_kv, d, m, seed=88, seq_lens=(700, 129))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    assert ek.decode_path(dw.shape) == ek.PATH_UNFUSED
    out, lse = dw.decode(); torch.cuda.synchronize()
    o_ref, l_ref = ref.decode_ref(inp)
    check(host(out), o_ref, "bf16", f"{w.name} decode on the materialising path")
    assert np.abs(host(lse) - l_ref).max() <= 2e-2


# ---- the paper's own (S, m) presets on its models' KV layout (8 KV heads x 128) ----------
# Appendix "Compression-Ratio Configurations": m = 384 (ratio 0.7), m = 0 (0.5), m = 64 (0.3;
# the retained prefix ends in the middle of head 0).  S only says how many target layers
# share an anchor; each (anchor, target) pair is one call.
@pytest.mark.parametrize("flags", MODES)
@pytest.mark.parametrize("m", [384, 0, 64, 192, 960])
def test_decode_paper_presets(m, flags):
    if flags & PACKED and m % 128:
        pytest.skip("packed weights are not offered when a head is split")
    w = synth.Workload(f"preset_m{m}", "bf16", 32, 8, 128, m, seed=50 + m, seq_lens=(700, 129))
    run_decode_case(w, flags)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_split_head_weights_extended_once(dtype):
    """echokv_augment_weights + ECHOKV_FLAG_W_AUGMENTED: the same kernels on the same extended
    weights as the per-call extension -> bit-equal decode (fused and unfused) and prefill."""
    w = synth.Workload("preset_m64_aug", dtype, 8, 4, 128, 64, seed=63, seq_lens=(300, 77),
                       prefill_len=260, prefill_q=200)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    tdt = dw.W_K.dtype
    n = ek.augmented_weight_elems(dw.shape)
    assert n == (512 + 64) * (512 - 64 + 64)
    wk_aug = torch.empty(n, dtype=tdt, device=dw.dev); wv_aug = torch.empty(n, dtype=tdt, device=dw.dev)
    ek.augment_weights(dw.shape, dw.W_K, dw.W_V, wk_aug, wv_aug); torch.cuda.synchronize()
    aug = wk_aug.view(512 + 64, 512).float().cpu().numpy()
    np.testing.assert_array_equal(aug[:, 64:], dw.W_K.float().cpu().numpy().reshape(512 + 64, 448))
    sel = np.zeros((512 + 64, 64), dtype=np.float32); sel[512 + np.arange(64), np.arange(64)] = 1.0
    np.testing.assert_array_equal(aug[:, :64], sel)
    for flags in (0, ek.FLAG_UNFUSED):
        dw.shape.flags = flags
        o0, l0 = dw.decode(); torch.cuda.synchronize()
        o0, l0 = host(o0).copy(), host(l0).copy()
        dw.shape.flags = flags | ek.FLAG_W_AUGMENTED
        ek.decode_attn(dw.shape, dw.anchor, dw.target, wk_aug, wv_aug, dw.q, dw.out, dw.lse, dw.workspace)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(host(dw.out), o0); np.testing.assert_array_equal(host(dw.lse), l0)
    dw.shape.flags = 0
    p0, pl0 = dw.prefill(); torch.cuda.synchronize()
    p0, pl0 = host(p0).copy(), host(pl0).copy()
    dw.shape.flags = ek.FLAG_W_AUGMENTED
    ek.prefill_attn(dw.shape, dw.anchor_all, dw.target_all, wk_aug, wv_aug, inp.n_decode, dw.q_prefill, 200,
                    inp.q_pos0, dw.out_prefill, dw.lse_prefill, dw.workspace)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host(dw.out_prefill), p0); np.testing.assert_array_equal(host(dw.lse_prefill), pl0)
    dw.shape.flags = 0


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_split_head_prefill_and_reconstruct(dtype):
    w = synth.Workload("preset_m64_pf", dtype, 8, 4, 128, 64, seed=61, seq_lens=(300,),
                       prefill_len=260, prefill_q=200)
    inp, dw = run_prefill_case(w)
    k_out, v_out = dw.reconstruct(0, 5, 290); torch.cuda.synchronize()
    k_ref, v_ref = ref.reconstruct_ref(inp, 0, 5, 290)
    assert np.array_equal(host(k_out)[:, :64], k_ref[:, :64])
    tol = 1e-5 if dtype == "f32" else 5e-3
    assert error_metrics(host(k_out), k_ref)[1] <= tol and error_metrics(host(v_out), v_ref)[1] <= tol
    run_decode_case(w.scaled(prefill_len=0, prefill_q=0), 0)
