"""GPU parity of decode with the one-hidden-layer predictor (Appendix "Prediction
Network Architecture") against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import echokv_oracle as orc
from paper_2603_22910_amd import binding as ek
from paper_2603_22910_amd import synth
from paper_2603_22910_amd.harness import DeviceWorkload, error_metrics

import oracle_ref as ref

pytestmark = pytest.mark.gpu
ACTS = [pytest.param(ek.ACT_RELU, "relu", id="relu"), pytest.param(ek.ACT_SILU, "silu", id="silu")]


def host(t):
    return t.float().cpu().numpy().astype(np.float64)


def run(w, hidden, act_code, act_name):
    inp = synth.generate(w)
    weights = synth.mlp_weights(w, hidden)
    dw = DeviceWorkload(inp)
    out, lse = dw.decode_mlp(weights, hidden, act_code)
    torch.cuda.synchronize()
    o_ref, l_ref = ref.decode_mlp_ref(inp, weights, act_name)
    mx, rl = error_metrics(host(out), o_ref)
    print(f"[parity] {w.name} mlp hidden={hidden} {act_name}: max_abs={mx:.3e} rel_l2={rl:.3e}", flush=True)
    assert np.isfinite(host(out)).all()
    assert mx <= 2e-2 and rl <= 5e-3
    assert np.abs(host(lse) - l_ref).max() <= 2e-2
    return inp, dw, weights


@pytest.mark.parametrize("act_code,act_name", ACTS)
@pytest.mark.parametrize("H_q,H_kv,d,m,hidden", [
    (8, 8, 128, 512, 1536),        # hidden = predictor input width (D + m)
    (8, 8, 128, 512, 384),         # parameter-matched width
    (32, 8, 128, 512, 1536),       # the paper's 8 x 128 GQA layout
    (32, 8, 128, 0, 512),          # ratio-0.5 preset (m = 0), parameter-matched
    (8, 4, 64, 128, 64),           # one k-tile of hidden units, head_dim 64
    (4, 4, 128, 512, 320),         # everything retained: the predictor is never run
])
def test_decode_mlp_shapes(H_q, H_kv, d, m, hidden, act_code, act_name):
    w = synth.Workload(f"mlp_{H_q}_{H_kv}_{d}_{m}_{hidden}", "bf16", H_q, H_kv, d, m,
                       seed=900 + hidden + m, seq_lens=(700, 129, 257, 1))
    run(w, hidden, act_code, act_name)


def test_param_matched_width_of_the_oracle_is_accepted():
    w = synth.CONFIGS[1].scaled(seq_lens=(513, 300))
    run(w, orc.mlp_param_matched_hidden(w.D, w.n_retained), ek.ACT_RELU, "relu")


def test_identity_first_layer_on_nonnegative_caches_equals_the_linear_predictor():
    """ReLU(x I) = x for x >= 0: the two-layer path then computes the linear predictor's
    function (its hidden activations are the stored bf16 values, exactly)."""
    w = synth.Workload("mlp_id", "bf16", 8, 4, 128, 256, seed=17, seq_lens=(400, 130))
    inp = synth.generate(w)
    for t in (inp.K_a, inp.V_a, inp.K_r, inp.V_r):
        t.abs_()
    eye = torch.eye(w.d_in, dtype=w.torch_dtype)
    dw = DeviceWorkload(inp)
    o_lin = host(dw.decode()[0]).copy(); torch.cuda.synchronize()
    o_mlp = host(dw.decode_mlp((eye, inp.W_K, eye, inp.W_V), w.d_in, ek.ACT_RELU)[0]); torch.cuda.synchronize()
    np.testing.assert_allclose(o_mlp, o_lin, rtol=0, atol=2e-3)
    o_ref, _ = ref.decode_ref(inp)
    mx, rl = error_metrics(o_mlp, o_ref)
    assert mx <= 2e-2 and rl <= 5e-3


def test_decode_mlp_more_sequences_than_one_launch():
    lens = tuple(1 + (41 * i) % 350 for i in range(135))
    w = synth.Workload("mlp_b135", "bf16", 4, 2, 128, 128, seed=5, seq_lens=lens)
    run(w, 128, ek.ACT_SILU, "silu")


def test_decode_mlp_argument_errors():
    w = synth.Workload("mlp_err", "bf16", 8, 4, 128, 256, seed=1, seq_lens=(100,))
    inp = synth.generate(w)
    dw = DeviceWorkload(inp)
    wts = synth.mlp_weights(w, 128)
    def code(hidden, act, shape=None):
        try:
            sh = shape or dw.shape
            ws = torch.empty(1 << 26, dtype=torch.uint8, device=dw.dev)
            d = [t.to(dw.dev) for t in wts]
            ek.decode_attn_mlp(sh, dw.anchor, dw.target, d[0], d[1], d[2], d[3], hidden, act, dw.q,
                               dw.out, dw.lse, ws)
        except ek.EchoKVError as e:
            return e.code
        return ek.OK
    assert code(100, ek.ACT_RELU) == ek.ERR_SHAPE          # hidden not a multiple of 64
    assert code(128, 7) == ek.ERR_SHAPE                    # unknown activation
    sh = ek.make_shape(8, 4, 128, 256, "bf16", flags=ek.FLAG_UNFUSED)
    assert code(128, ek.ACT_RELU, sh) == ek.ERR_UNSUPPORTED
    sh64 = ek.make_shape(8, 4, 128, 64, "bf16")            # retained prefix ends inside a head
    assert ek.mlp_workspace_bytes(sh64, 1, 100, 128) == 0
    assert code(128, ek.ACT_RELU) == ek.OK
    torch.cuda.synchronize()
