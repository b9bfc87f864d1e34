"""GPU parity of the LRPE-d rotation kernels and of the whole LRPE-d attention layer
(rotate -> wide attention -> its backward -> rotation backward) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2405_17381_amd import binding

pytestmark = pytest.mark.gpu
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def _np(t):
    return t.to(torch.float64).cpu().numpy()


@pytest.mark.parametrize("dtype,B,H,n,d", [("f32", 2, 3, 300, 64), ("f32", 1, 2, 129, 128), ("bf16", 2, 4, 1000, 128),
                                            ("bf16", 1, 5, 77, 64), ("f32", 1, 1, 1, 64), ("f32", 1, 2, 70000, 64)])
def test_rotation_forward_and_backward(dtype, B, H, n, d):
    g = torch.Generator(device="cpu").manual_seed(8000 + n + d)
    X = torch.randn((B, H, n, d), generator=g).to(TDT[dtype])
    G = torch.randn((B, H, n, 2 * d), generator=g).to(TDT[dtype])
    theta = torch.rand((H, d), generator=g) * 2.0                # angles up to 2 rad per position
    Xw = binding.la_lrpe_rotate_fwd(X.cuda(), theta.cuda())
    dX, dth = binding.la_lrpe_rotate_bwd(X.cuda(), theta.cuda(), G.cuda())
    dX2, dth2 = binding.la_lrpe_rotate_bwd(X.cuda(), theta.cuda(), G.cuda(), dtheta=dth.clone(), accumulate=True)
    torch.cuda.synchronize()
    x, gg, th = _np(X), _np(G), _np(theta)
    ref_w = oracle.lrpe_features(x, th)
    ref_dx, ref_dth = oracle.lrpe_features_bwd(x, th, gg)
    # fp32: the error is that of the hardware sin / cos (about 1e-6 of a revolution); bf16: one rounding
    tol = 2e-5 if dtype == "f32" else 8e-3
    assert oracle.rel_max_err(_np(Xw), ref_w) <= tol
    assert oracle.rel_max_err(_np(dX), ref_dx) <= tol
    assert oracle.rel_max_err(_np(dth), ref_dth) <= (1e-4 if dtype == "f32" else 2e-2)
    assert np.array_equal(_np(dX2), _np(dX))
    assert oracle.rel_max_err(_np(dth2), 2.0 * ref_dth) <= (1e-4 if dtype == "f32" else 2e-2)


@pytest.mark.parametrize("dtype,n,d", [("f32", 200, 64), ("bf16", 900, 128)])
def test_lrpe_d_layer_forward_and_backward(dtype, n, d):
    """Everything on the GPU: rotate Q and K, wide attention, its backward, rotation backward.
    Reference: the oracle's chain, whose forward is pinned to LRPE-d's definition."""
    B, H = 2, 3
    lam = [1.0, 0.98, 0.9]
    g = torch.Generator(device="cpu").manual_seed(8100 + n)
    Q, K, V = [(torch.randn((B, H, n, d), generator=g) / d ** 0.5).to(TDT[dtype]) for _ in range(3)]
    dO = torch.randn((B, H, n, d), generator=g).to(TDT[dtype])
    theta = torch.rand((H, d), generator=g)
    Qd, Kd, Vd, dOd, thd = [x.cuda() for x in (Q, K, V, dO, theta)]
    Qw = binding.la_lrpe_rotate_fwd(Qd, thd)
    Kw = binding.la_lrpe_rotate_fwd(Kd, thd)
    O = binding.la_fwd_wide(Qw, Kw, Vd, lam)
    dQw, dKw, dV = binding.la_bwd_wide(Qw, Kw, Vd, lam, dOd)
    dQ, dth = binding.la_lrpe_rotate_bwd(Qd, thd, dQw)
    dK, dth = binding.la_lrpe_rotate_bwd(Kd, thd, dKw, dtheta=dth, accumulate=True)
    torch.cuda.synchronize()

    q, k, v, go, th = [_np(x) for x in (Q, K, V, dO, theta)]
    qw, kw = oracle.lrpe_features(q, th), oracle.lrpe_features(k, th)
    O_r = oracle.recurrence_fwd(qw, kw, v, lam)
    dqw, dkw, dV_r = oracle.recurrence_bwd(qw, kw, v, lam, go)
    dQ_r, dth_q = oracle.lrpe_features_bwd(q, th, dqw)
    dK_r, dth_k = oracle.lrpe_features_bwd(k, th, dkw)
    if n <= 200:                                   # the definition itself, term by term
        assert oracle.rel_max_err(O_r, oracle.lrpe_fwd(q, k, v, lam, th)) <= 1e-12
    tol = 1e-4 if dtype == "f32" else 2e-2
    for nm, x, r in (("O", O, O_r), ("dQ", dQ, dQ_r), ("dK", dK, dK_r), ("dV", dV, dV_r)):
        assert oracle.rel_max_err(_np(x), r) <= tol, nm
    # theta's gradient sums position-weighted terms over all tokens: looser in bf16
    assert oracle.rel_max_err(_np(dth), dth_q + dth_k) <= (2e-4 if dtype == "f32" else 3e-2)
