"""The decode and prefill entry points allocate nothing, synchronise nothing and clear nothing with
memsets, so a caller may capture them in a HIP graph.  Each replay is checked against an
eager call on the same inputs, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags", [pytest.param(0, id="fused"), pytest.param(ek.FLAG_ABSORBED, id="absorbed"),
                                   pytest.param(ek.FLAG_ABSORB_V, id="absorb_v"),
                                   pytest.param(ek.FLAG_UNFUSED, id="unfused")])
def test_decode_in_a_captured_graph_matches_eager_on_every_replay(flags):
    w = synth.Workload("graph", "bf16", 8, 4, 128, 256, seed=61, seq_lens=(700, 129, 300))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp, flags=flags)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        dw.decode(stream=side.cuda_stream)          # warm-up on the capture stream
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        dw.decode(stream=torch.cuda.current_stream().cuda_stream)
    gen = torch.Generator().manual_seed(3)
    for rep in range(4):
        q_new = torch.randn(dw.q.shape, generator=gen).to(dw.q.dtype)
        dw.q.copy_(q_new.to(dw.dev))                # same buffer the graph reads
        torch.cuda.synchronize()
        dw.out.zero_(); dw.lse.zero_()
        g.replay()
        torch.cuda.synchronize()
        got, got_lse = dw.out.clone(), dw.lse.clone()
        dw.out.zero_(); dw.lse.zero_()
        dw.decode()                                  # eager, default stream
        torch.cuda.synchronize()
        assert torch.equal(got, dw.out), (flags, rep)
        assert torch.equal(got_lse, dw.lse), (flags, rep)
        assert float(got.float().abs().sum()) > 0


@pytest.mark.parametrize("pq,use_rope,ctx", [
    pytest.param(300, False, 211, id="short"), pytest.param(1100, False, 211, id="long"),
    pytest.param(1100, True, 211, id="long+rope"),
    pytest.param(300, False, 2500, id="short-behind-long-context"),       # split over the keys + merge kernel
    pytest.param(300, True, 2500, id="short-behind-long-context+rope")])
def test_prefill_in_a_captured_graph_matches_eager_on_every_replay(pq, use_rope, ctx):
    """The prefill attention kernels (and the key rotation ahead of them).  The first call on
    a device sets a function attribute of the long-chunk kernel: it runs before the capture."""
    w = synth.Workload("graph_pf", "bf16", 8, 4, 128, 256, seed=62, seq_lens=(5,), prefill_len=pq + ctx,
                       prefill_q=pq)
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    rope = tuple(t.to(dw.dev) for t in synth.rope_tables(128, pq + ctx + 89)) if use_rope else None
    run = (lambda st=None: dw.prefill_ex(rope, stream=st)) if use_rope else (lambda st=None: dw.prefill(stream=st))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        run(side.cuda_stream)
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        run(torch.cuda.current_stream().cuda_stream)
    gen = torch.Generator().manual_seed(4)
    for rep in range(3):
        q_new = torch.randn(dw.q_prefill.shape, generator=gen).to(dw.q_prefill.dtype)
        dw.q_prefill.copy_(q_new.to(dw.dev))
        torch.cuda.synchronize()
        dw.out_prefill.zero_(); dw.lse_prefill.zero_()
        g.replay()
        torch.cuda.synchronize()
        got, got_lse = dw.out_prefill.clone(), dw.lse_prefill.clone()
        dw.out_prefill.zero_(); dw.lse_prefill.zero_()
        run()
        torch.cuda.synchronize()
        assert torch.equal(got, dw.out_prefill), rep
        assert torch.equal(got_lse, dw.lse_prefill), rep
        assert float(got.float().abs().sum()) > 0


def test_stream_read_yardstick_runs_and_is_plausible():
    buf = torch.ones(1 << 29, dtype=torch.uint8, device="cuda:0")
    rate = ek.profile_stream_read(buf, 3)
    assert 1000.0 < rate < 8000.0        # GB/s: above any PCIe-like figure, below the nominal HBM peak
    with pytest.raises(ek.EchoKVError):
        ek.profile_stream_read(torch.ones(1 << 20, dtype=torch.uint8, device="cuda:0"), 3)   # too small
