"""GPU check of the closed-form predictor fit (stage-1 reconstruction loss) against the
fp64 least-squares oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import echokv_oracle as orc
from paper_2603_22910_amd import binding as ek

pytestmark = pytest.mark.gpu


def make_rows(T, D, m, noise, seed):
    """Anchor rows ~ N(0,1); the target's full rows = [anchor ; noise-free mix] (so that its
    dropped dims are predictable from the inputs up to `noise`), rounded to bf16."""
    g = torch.Generator().manual_seed(seed)
    A = torch.randn(T, D, generator=g)
    M = torch.randn(D, D, generator=g) / math.sqrt(D)
    Tt = A @ M + noise * torch.randn(T, D, generator=g)
    return A.to(torch.bfloat16), Tt.to(torch.bfloat16)


@pytest.mark.parametrize("H_kv,d,m,T,noise,ridge", [
    (4, 128, 256, 4096, 0.1, 0.0),
    (4, 128, 0, 2048, 0.3, 0.0),        # no local input
    (8, 64, 192, 3072, 0.2, 5.0),       # ridge
    (2, 128, 64, 1024, 0.05, 0.0),      # retained prefix ends inside a head
])
def test_fit_linear_matches_least_squares(H_kv, d, m, T, noise, ridge):
    D = H_kv * d
    A, Tt = make_rows(T, D, m, noise, seed=H_kv * 1000 + m)
    sh = ek.make_shape(H_kv, H_kv, d, m, "bf16")
    dev = torch.device("cuda:0")
    need = ek.fit_workspace_bytes(sh, T)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    w_out = torch.empty(D + m, D - m, dtype=torch.bfloat16, device=dev)
    iters, res = ek.fit_linear(sh, A.to(dev), Tt.to(dev), T, w_out, ws, ridge=ridge, max_iters=300, tol=1e-6)
    torch.cuda.synchronize()
    print(f"[fit] D={D} m={m} T={T}: {iters} CG steps, relative residual {res:.2e}", flush=True)
    assert res <= 1e-5
    A64, T64 = A.double().numpy(), Tt.double().numpy()
    W_ref = orc.fit_linear(A64, T64, m, ridge=ridge)
    W_got = w_out.float().cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(W_got - W_ref) / np.linalg.norm(W_ref)
    loss_ref = orc.reconstruction_loss(A64, T64, m, W_ref)
    loss_got = orc.reconstruction_loss(A64, T64, m, W_got)
    print(f"[fit] |W - W_ref| / |W_ref| = {rel:.3e}; loss {loss_got:.6e} vs optimum {loss_ref:.6e}", flush=True)
    assert rel <= 5e-3                       # the bf16 rounding of the result is 2^-9 per entry
    assert loss_got <= loss_ref * 1.02 + 1e-6


def test_fit_then_decode_uses_the_fitted_weights():
    """Fit W_K, W_V on synthetic rows, then decode with them: the attention output is close to
    attention over the target layer's true rows (what the compression is meant to preserve)."""
    from paper_2603_22910_amd import synth
    from paper_2603_22910_amd.harness import DeviceWorkload
    w = synth.Workload("fit_dec", "bf16", 8, 4, 128, 256, seed=31, seq_lens=(1024,))
    inp = synth.generate(w)
    D, m, T = w.D, w.n_retained, 1024
    dev = torch.device("cuda:0")
    g = torch.Generator().manual_seed(5)
    full = {}
    for tag, A, R in (("K", inp.K_a, inp.K_r), ("V", inp.V_a, inp.V_r)):
        M2 = torch.randn(D, D - m, generator=g) / math.sqrt(D)
        drop = (A[:T].float() @ M2 + 0.05 * torch.randn(T, D - m, generator=g)).to(torch.bfloat16)
        full[tag] = torch.cat([R[:T], drop], dim=1).contiguous()
    sh = ek.make_shape(w.n_q_heads, w.n_kv_heads, w.head_dim, m, "bf16")
    ws = torch.empty(ek.fit_workspace_bytes(sh, T), dtype=torch.uint8, device=dev)
    fitted = {}
    for tag, A in (("K", inp.K_a), ("V", inp.V_a)):
        wt = torch.empty(w.d_in, w.d_out, dtype=torch.bfloat16, device=dev)
        ek.fit_linear(sh, A[:T].to(dev), full[tag].to(dev), T, wt, ws, max_iters=300, tol=1e-6)
        fitted[tag] = wt.cpu()
    inp.W_K, inp.W_V = fitted["K"], fitted["V"]
    dw = DeviceWorkload(inp)
    out = dw.decode()[0].float().cpu().numpy().astype(np.float64); torch.cuda.synchronize()
    o_true, _, _ = orc.attention_rows(inp.q[:1].double().numpy(), full["K"].double().numpy(),
                                      full["V"].double().numpy(), w.n_kv_heads)
    err = np.linalg.norm(out[0] - o_true[0]) / np.linalg.norm(o_true[0])
    print(f"[fit] decode with fitted predictors vs attention over the true rows: rel-L2 {err:.3e}", flush=True)
    assert err < 0.1
