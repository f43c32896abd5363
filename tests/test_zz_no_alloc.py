"""echokv_decode_attn_static (the entry point for callers that cannot allocate: it runs on the
library's fixed scratch instead of a workspace) against echokv_decode_attn on the same inputs:
the same kernels in the same order, so the outputs must be bit-identical.  Two calls in a row, the
second on a smaller input, so whatever the first call left in the scratch is still there."""
import numpy as np
import pytest
import torch

from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload, error_metrics

import oracle_ref as ref

pytestmark = pytest.mark.gpu


def both_ways(w, flags=0):
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, flags=flags)
    out_ws, lse_ws = dw.decode()
    torch.cuda.synchronize()
    out_ws, lse_ws = out_ws.clone(), lse_ws.clone()
    out_st = torch.full_like(dw.out, float("nan"))
    lse_st = torch.full_like(dw.lse, float("nan"))
    ek.decode_attn_static(dw.shape, dw.anchor, dw.target, dw.W_K, dw.W_V, dw.q, out_st, lse_st)
    torch.cuda.synchronize()
    print(f"[static] {w.name} flags={flags}: {inp.total_decode_tokens} tokens", flush=True)
    assert torch.equal(out_st.view(torch.int16), out_ws.view(torch.int16))
    assert torch.equal(lse_st.view(torch.int32), lse_ws.view(torch.int32))
    return inp, out_st


@pytest.mark.parametrize("flags", [0, ek.FLAG_ABSORBED, ek.FLAG_UNFUSED], ids=["fused", "absorbed", "unfused"])
def test_static_scratch_matches_workspace_call_twice_in_a_row(flags):
    # the unfused path also keeps K-hat / V-hat of every token in the scratch: fewer tokens fit
    big = synth.CONFIGS[1].scaled(seq_lens=(1500, 513, 1) if flags & ek.FLAG_UNFUSED else (3000, 1700, 513, 1))
    small = synth.CONFIGS[1].scaled(seq_lens=(300, 129))
    both_ways(big, flags)
    inp, out = both_ways(small, flags)            # second call, smaller input, scratch left dirty
    o_ref, _ = ref.decode_ref(inp)
    mx, rl = error_metrics(out.float().cpu().double().numpy(), o_ref)
    assert mx <= 2e-2 and rl <= 5e-3


def test_static_scratch_split_head_and_gqa():
    # the half-head preset keeps extended weights in the scratch as well
    w = synth.Workload("static_split_head", "bf16", 32, 8, 128, 64, seed=11, seq_lens=(2000, 700))
    both_ways(w)
    both_ways(synth.Workload("static_split_head_small", "bf16", 32, 8, 128, 64, seed=12, seq_lens=(130,)))


def test_static_scratch_limit_is_an_error_and_touches_nothing():
    # the unfused path keeps K-hat / V-hat of every token in its workspace: far beyond the limit here
    w = synth.CONFIGS[1].scaled(seq_lens=(40000,))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, flags=ek.FLAG_UNFUSED)
    out = torch.full_like(dw.out, 7.0)
    with pytest.raises(ek.EchoKVError) as e:
        ek.decode_attn_static(dw.shape, dw.anchor, dw.target, dw.W_K, dw.W_V, dw.q, out, dw.lse)
    assert e.value.code == ek.ERR_STATIC_LIMIT
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # argument errors come first, as everywhere
    with pytest.raises(ek.EchoKVError) as e:
        ek.decode_attn_static(dw.shape, dw.anchor, dw.target, dw.W_K, dw.W_V, None, out, dw.lse)
    assert e.value.code == ek.ERR_NULL
