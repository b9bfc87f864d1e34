"""GPU parity of the attention with a query / key feature wider than the value feature
(la_fwd_wide, la_bwd_wide), and of LRPE-d served through it, against the CPU oracle."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2405_17381_amd import binding

pytestmark = pytest.mark.gpu
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _draw(B, H, n, dk, dv, dtype, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    Qw = torch.randn((B, H, n, dk), generator=g) / dk ** 0.5
    Kw = torch.randn((B, H, n, dk), generator=g) / dk ** 0.5
    V = torch.randn((B, H, n, dv), generator=g) / dv ** 0.5
    dO = torch.randn((B, H, n, dv), generator=g)
    return [x.to(TDT[dtype]) for x in (Qw, Kw, V, dO)]


def _run(xs, lam, lseg):
    if lseg is not None:
        binding.debug_set("lseg", lseg)
    try:
        Qw, Kw, V, dO = [x.cuda() for x in xs]
        O = binding.la_fwd_wide(Qw, Kw, V, lam)
        dQw, dKw, dV = binding.la_bwd_wide(Qw, Kw, V, lam, dO)
        torch.cuda.synchronize()
    finally:
        binding.debug_set("lseg", 0)
    return [t.to(torch.float64).cpu().numpy() for t in (O, dQw, dKw, dV)]


def _reference(xs, lam):
    """The compiled recurrence handles square states: use the slice-sum identity the oracle's
    pins establish (scores add over the slices of d_v features)."""
    qw, kw, v, g = [x.to(torch.float64).numpy() for x in xs]
    dv = v.shape[3]
    m = qw.shape[3] // dv
    O = np.zeros_like(v)
    dQw, dKw, dV = np.empty_like(qw), np.empty_like(kw), np.zeros_like(v)
    for j in range(m):
        sl = slice(j * dv, (j + 1) * dv)
        q, k = np.ascontiguousarray(qw[..., sl]), np.ascontiguousarray(kw[..., sl])
        O += oracle.c_recurrence_fwd(q, k, v, lam)
        a, b, c = oracle.c_recurrence_bwd(q, k, v, lam, g)
        dQw[..., sl], dKw[..., sl] = a, b
        dV += c
    return O, dQw, dKw, dV


@pytest.mark.parametrize("dtype,B,H,n,dk,dv,lseg", [
    ("f32", 1, 2, 300, 128, 64, None), ("f32", 2, 2, 200, 128, 64, 64), ("f32", 1, 2, 150, 256, 128, None),
    ("bf16", 2, 4, 1000, 256, 128, None), ("bf16", 2, 4, 1000, 256, 128, 256), ("bf16", 1, 3, 1, 256, 128, None),
    ("bf16", 2, 3, 700, 128, 64, None), ("bf16", 2, 3, 700, 192, 64, 192), ("bf16", 1, 2, 333, 128, 128, None),
    ("bf16", 1, 16, 4096, 256, 128, 1024),
    # whole sequences at d_k = 256, d_v = 128 in bf16: the forward pass is ONE kernel with the 256 x 128 state
    ("bf16", 2, 4, 500, 256, 128, None), ("bf16", 1, 3, 333, 256, 128, None), ("bf16", 16, 16, 1100, 256, 128, None),
])
def test_wide_attention_against_oracle(dtype, B, H, n, dk, dv, lseg):
    assert torch.cuda.is_available()
    lam = [1.0, 0.999, 0.97, 0.9][:H] if H <= 4 else list(np.linspace(0.9, 1.0, H))
    xs = _draw(B, H, n, dk, dv, dtype, seed=6000 + n + dk)
    got = _run(xs, lam, lseg)
    ref = _reference(xs, lam)
    for nm, x, r in zip(("O", "dQw", "dKw", "dV"), got, ref):
        assert np.all(np.isfinite(x)), nm
        err = oracle.rel_max_err(x, r)
        assert err <= TOL[dtype], (nm, err)


def test_single_kernel_and_sliced_wide_forward_agree():
    """d_k = 256, d_v = 128, one segment: la_fwd_wide runs the kernel that holds the whole non-square
    state; the "wide_slices" switch forces the two accumulated scans.  Same result up to rounding (the
    sliced path rounds O to bf16 between the slices), both within tolerance of the oracle, and they
    are different code."""
    lam = [1.0, 0.999, 0.97, 0.9]
    xs = _draw(8, 4, 512, 256, 128, "bf16", seed=77)
    assert binding.la_plan(8, 4, 512, 128, binding.LA_BF16)[2] == 1
    Qw, Kw, V, _ = [x.cuda() for x in xs]
    one = binding.la_fwd_wide(Qw, Kw, V, lam)
    with binding.debug(wide_slices=1):
        two = binding.la_fwd_wide(Qw, Kw, V, lam)
    torch.cuda.synchronize()
    ref = _reference(xs, lam)[0]
    a, b = one.double().cpu().numpy(), two.double().cpu().numpy()
    assert oracle.rel_max_err(a, ref) <= TOL["bf16"] and oracle.rel_max_err(b, ref) <= TOL["bf16"]
    assert oracle.rel_max_err(a, b) <= 1e-2 and not np.array_equal(a, b)
    print("  single kernel err %.3e, sliced err %.3e" % (oracle.rel_max_err(a, ref), oracle.rel_max_err(b, ref)), flush=True)


def test_small_case_against_the_quadratic_form():
    """No slice-sum identity in the reference: the oracle's quadratic form takes the wide operands as they are."""
    lam = [0.9, 1.0]
    xs = _draw(1, 2, 96, 128, 64, "f32", seed=61)
    got = _run(xs, lam, None)
    qw, kw, v, g = [x.to(torch.float64).numpy() for x in xs]
    ref = (oracle.left_product_fwd(qw, kw, v, lam),) + oracle.left_product_bwd(qw, kw, v, lam, g)
    for nm, x, r in zip(("O", "dQw", "dKw", "dV"), got, ref):
        assert oracle.rel_max_err(x, r) <= 1e-4, nm


def test_lrpe_d_through_the_wide_entry_point():
    """LRPE-d: rotate q and k into cos / sin features (here on the host, in fp64), run the wide
    attention on the GPU, compare with the definition written out term by term."""
    B, H, n, d = 1, 2, 80, 64
    lam = [0.95, 1.0]
    rng = np.random.default_rng(5)
    theta = rng.uniform(0.0, 1.0, size=(H, d))
    Q, K, V = (rng.standard_normal((B, H, n, d)) / d ** 0.5 for _ in range(3))
    Qw = torch.from_numpy(oracle.lrpe_features(Q, theta)).float().cuda()
    Kw = torch.from_numpy(oracle.lrpe_features(K, theta)).float().cuda()
    O = binding.la_fwd_wide(Qw, Kw, torch.from_numpy(V).float().cuda(), lam)
    torch.cuda.synchronize()
    ref = oracle.lrpe_fwd(Q, K, V, lam, theta)
    assert oracle.rel_max_err(O.double().cpu().numpy(), ref) <= 1e-4


def test_dk_equal_dv_is_the_plain_attention_bit_for_bit():
    """One slice of the full width: the wide entry points run the plain attention's kernels with an
    explicit row stride, in either kernel family of bf16 at d = 128."""
    lam = [0.99, 0.9]
    xs = _draw(2, 2, 500, 128, 128, "bf16", seed=62)
    Q, K, V, dO = [x.cuda() for x in xs]
    for staged in (0, 1):
        with binding.debug(staged_scan=staged):
            wide = _run(xs, lam, None)
            O = binding.la_fwd(Q, K, V, lam)
            dQ, dK, dV = binding.la_bwd(Q, K, V, lam, dO)
            torch.cuda.synchronize()
        for a, b in zip(wide, (O, dQ, dK, dV)):
            assert np.array_equal(a, b.double().cpu().numpy()), "staged_scan=%d" % staged
