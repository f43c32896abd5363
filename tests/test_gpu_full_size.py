"""The benchmark's configurations 1-4 at FULL size, in the launch configuration bench.py times,
against the fp64 oracle: every sequence, every head, every output element (relative L2 error over
the whole output tensor of the configuration, maximum absolute error over every element, and the
log-sum-exp of every (sequence, head)).  Decode runs in the fused and in the weight-absorbed mode on
the same inputs; the 8192-query causal prefill chunk of configuration 4 is checked on all of its
rows, the oracle's attention evaluated in blocks of query rows so that its probability tensor
stays small."""
import gc

import numpy as np
import pytest
import torch

from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload, error_metrics

import oracle_ref as ref

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, LSE_ABS = 2e-2, 5e-3, 2e-2


def host(t):
    return t.float().cpu().double().numpy()


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_decode_full_size_every_element(cfg):
    w = synth.CONFIGS[cfg]
    if cfg == 4:                      # the chunk has its own test below
        w = w.scaled(prefill_len=0, prefill_q=0)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, flags=ek.FLAG_ABSORBED)      # workspace sized for both paths
    results = {}
    for name, fl in (("fused", 0), ("absorbed", ek.FLAG_ABSORBED)):
        dw.set_flags(fl)
        out, lse = dw.decode(); torch.cuda.synchronize()
        results[name] = (host(out).copy(), host(lse).copy())
    del dw
    gc.collect(); torch.cuda.empty_cache()
    o_ref, l_ref = ref.decode_ref(inp)                    # every sequence, every head
    assert o_ref.shape == (inp.n_decode, w.n_q_heads, w.head_dim)
    for name, (got, got_lse) in results.items():
        assert np.isfinite(got).all() and np.isfinite(got_lse).all()
        mx, rl = error_metrics(got, o_ref)
        worst_row = max(error_metrics(got[b, h], o_ref[b, h])[1]
                        for b in range(inp.n_decode) for h in range(w.n_q_heads))
        lse_err = float(np.abs(got_lse - l_ref).max())
        print(f"[full] {w.name} {name}: {inp.total_decode_tokens} tokens, {inp.n_decode} sequences: "
              f"max_abs={mx:.3e} rel_l2={rl:.3e} worst (seq, head) rel_l2={worst_row:.3e} "
              f"lse max_abs={lse_err:.3e}", flush=True)
        assert mx <= MAX_ABS and rl <= REL_L2, (name, mx, rl)
        assert lse_err <= LSE_ABS, (name, lse_err)


@pytest.mark.parametrize("q_pos0", [0, 3000])
def test_prefill_full_size_every_row(q_pos0):
    """The benchmark's 8192-query causal chunk on the 7B-shaped layer (50 % retention): all rows,
    all heads.  q_pos0 = 0 is the benchmark's chunk; 3000 puts cached context in front of it."""
    from oracle import echokv_oracle as orc
    T_q, QB = 8192, 256
    w = synth.CONFIGS[4].scaled(batch=0, seq_lens=(300,), prefill_len=q_pos0 + T_q, prefill_q=T_q)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    out, lse = dw.prefill(); torch.cuda.synchronize()
    got, got_lse = host(out), host(lse)
    assert np.isfinite(got).all() and np.isfinite(got_lse).all()
    b = inp.n_decode
    K_a, V_a, K_r, V_r = ref.seq_arrays(inp, b)
    W_K, W_V = ref.weights(inp)
    K_t = orc.reconstruct(K_a, K_r, W_K); V_t = orc.reconstruct(V_a, V_r, W_V)   # Eq. 3, 6 once
    Q = ref.f64(inp.q_prefill)
    o_ref = np.empty_like(got); l_ref = np.empty_like(got_lse)
    for i0 in range(0, T_q, QB):                  # Eq. 7 with the causal mask, 256 query rows at a time
        i1 = min(T_q, i0 + QB)
        end = q_pos0 + i1                          # no row of the block sees further
        o, l, _ = orc.attention_rows(Q[i0:i1], K_t[:end], V_t[:end], w.n_kv_heads,
                                     visible=[q_pos0 + i + 1 for i in range(i0, i1)])
        o_ref[i0:i1] = o; l_ref[i0:i1] = l
    mx, rl = error_metrics(got, o_ref)
    lse_err = float(np.abs(got_lse - l_ref).max())
    print(f"[full] prefill chunk {T_q} queries at q_pos0={q_pos0}: max_abs={mx:.3e} rel_l2={rl:.3e} "
          f"lse max_abs={lse_err:.3e}", flush=True)
    assert mx <= MAX_ABS and rl <= REL_L2
    assert lse_err <= LSE_ABS
