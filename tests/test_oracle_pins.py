"""Pins for the CPU oracle: it is checked against things other than itself.

The paper prints no numeric worked example, so the pins are: hand-worked tiny
cases (tests/golden), closed forms, textbook special cases, the agreement of
the two independent forms (App. A proves them equal), finite differences,
a blocked re-statement of Alg. 5/6 (App. C proves block form == token form),
the trilinearity invariant and causality.
"""
import math

import numpy as np
import pytest

import oracle
from conftest import load_golden

LAMS = [1.0, 0.99, 0.5, 0.1]


def _rand(B, H, n, d, seed):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((B, H, n, d)) for _ in range(4)]


FWD_IMPLS = {
    "left": oracle.left_product_fwd,
    "rec": oracle.recurrence_fwd,
    "c_rec": oracle.c_recurrence_fwd,
}
BWD_IMPLS = {
    "left": oracle.left_product_bwd,
    "rec": oracle.recurrence_bwd,
    "c_rec": oracle.c_recurrence_bwd,
}


# ---- 1. hand-worked examples ------------------------------------------------
@pytest.mark.parametrize("fixture", ["worked_example_a.txt", "worked_example_b.txt"])
@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_worked_examples(fixture, impl):
    g = load_golden(fixture)
    lam = [g["lambda"]]
    O = FWD_IMPLS[impl](g["Q"], g["K"], g["V"], lam)
    dQ, dK, dV = BWD_IMPLS[impl](g["Q"], g["K"], g["V"], lam, g["dO"])
    np.testing.assert_allclose(O, g["O"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dQ, g["dQ"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dK, g["dK"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(dV, g["dV"], rtol=0, atol=1e-13)


# ---- 2. the two forms agree (App. A induction) -------------------------------
@pytest.mark.parametrize("n,d", [(1, 3), (5, 2), (17, 8), (64, 8)])
def test_forms_agree(n, d):
    Q, K, V, dO = _rand(2, len(LAMS), n, d, seed=n * 100 + d)
    ref_o = oracle.left_product_fwd(Q, K, V, LAMS)
    ref_g = oracle.left_product_bwd(Q, K, V, LAMS, dO)
    for name in ("rec", "c_rec"):
        o = FWD_IMPLS[name](Q, K, V, LAMS)
        assert oracle.rel_max_err(o, ref_o) < 1e-12, name
        for x, r in zip(BWD_IMPLS[name](Q, K, V, LAMS, dO), ref_g):
            assert oracle.rel_max_err(x, r) < 1e-12, name


# ---- 3. closed form: all-ones inputs -----------------------------------------
@pytest.mark.parametrize("lam", LAMS)
@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_all_ones_closed_form(lam, impl):
    n, d = 23, 5
    X = np.ones((1, 1, n, d))
    O = FWD_IMPLS[impl](X, X, X, [lam])
    t = np.arange(1, n + 1, dtype=np.float64)
    # o_t[j] = sum_{s<=t} lam^(t-s) * (q_t.k_s) * v_s[j] = d * sum_{m=0}^{t-1} lam^m
    expect = d * t if lam == 1.0 else d * (1 - lam ** t) / (1 - lam)
    np.testing.assert_allclose(O[0, 0], np.repeat(expect[:, None], d, axis=1), rtol=1e-12)


# ---- 4. textbook special cases -----------------------------------------------
@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_lambda_one_is_tril_gemm(impl):
    Q, K, V, dO = _rand(1, 1, 19, 6, seed=7)
    O = FWD_IMPLS[impl](Q, K, V, [1.0])
    expect = np.tril(Q[0, 0] @ K[0, 0].T) @ V[0, 0]
    np.testing.assert_allclose(O[0, 0], expect, rtol=1e-11, atol=1e-12)
    # last row is the plain (non-causal) right product q_n^T (K^T V)
    np.testing.assert_allclose(O[0, 0, -1], Q[0, 0, -1] @ (K[0, 0].T @ V[0, 0]),
                               rtol=1e-11, atol=1e-12)
    dQ, dK, dV = BWD_IMPLS[impl](Q, K, V, [1.0], dO)
    Gm = np.tril(dO[0, 0] @ V[0, 0].T)
    Pm = np.tril(Q[0, 0] @ K[0, 0].T)
    np.testing.assert_allclose(dQ[0, 0], Gm @ K[0, 0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dK[0, 0], Gm.T @ Q[0, 0], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dV[0, 0], Pm.T @ dO[0, 0], rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_single_token_and_vanishing_lambda(impl):
    Q, K, V, dO = _rand(1, 1, 1, 4, seed=3)
    O = FWD_IMPLS[impl](Q, K, V, [0.7])
    np.testing.assert_allclose(O[0, 0, 0], (Q[0, 0, 0] @ K[0, 0, 0]) * V[0, 0, 0], rtol=1e-13)
    # lam -> 0+: only the diagonal survives: o_t = (q_t.k_t) v_t
    Q, K, V, dO = _rand(1, 1, 9, 4, seed=4)
    O = FWD_IMPLS[impl](Q, K, V, [1e-300])
    expect = np.sum(Q[0, 0] * K[0, 0], axis=1, keepdims=True) * V[0, 0]
    np.testing.assert_allclose(O[0, 0], expect, rtol=1e-12, atol=1e-290)


# ---- 5. trilinearity: <dO,O> = <dQ,Q> = <dK,K> = <dV,V> -----------------------
@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_trilinearity_invariant(impl):
    Q, K, V, dO = _rand(2, 4, 16, 4, seed=11)
    O = FWD_IMPLS[impl](Q, K, V, LAMS)
    dQ, dK, dV = BWD_IMPLS[impl](Q, K, V, LAMS, dO)
    base = np.sum(dO * O)
    for g, x in ((dQ, Q), (dK, K), (dV, V)):
        assert abs(np.sum(g * x) - base) <= 1e-11 * abs(base)


# ---- 6. finite differences (fp64, n <= 16) ------------------------------------
@pytest.mark.parametrize("impl", list(BWD_IMPLS))
def test_finite_differences(impl):
    B, H, n, d = 1, 2, 12, 3
    lam = [0.9, 1.0]
    Q, K, V, dO = _rand(B, H, n, d, seed=21)
    dQ, dK, dV = BWD_IMPLS[impl](Q, K, V, lam, dO)
    fwd = oracle.left_product_fwd

    def loss(q, k, v):
        return float(np.sum(dO * fwd(q, k, v, lam)))

    eps = 1e-6
    rng = np.random.default_rng(5)
    for which, grad in ((0, dQ), (1, dK), (2, dV)):
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in (B, H, n, d))
            args_p = [Q.copy(), K.copy(), V.copy()]
            args_m = [Q.copy(), K.copy(), V.copy()]
            args_p[which][idx] += eps
            args_m[which][idx] -= eps
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), (which, idx)


# ---- 7. block form == token form (App. C's block identities) -------------------
def _block_identities(Q, K, V, lam, dO, Bk, lambda_from_zero=False):
    """The decomposition that Alg. 5 / Alg. 6 rest on (App. C), evaluated block by block with no
    running update at all.  For the block of rows [t0, t1):
      * the intra part is the oracle's quadratic form applied to the block alone;
      * the state entering from the left and the one entering from the right are written
        out as explicit weighted sums over the tokens outside the block,
            KV  = sum_{s <  t0} lam^(t0-1-s) k_s v_s^T      (nearest earlier token: weight 1)
            dKV = sum_{s >= t1} lam^(s-t1+1) q_s do_s^T     (nearest later token: weight lam);
      * row r = 1..Bk of the block sees KV scaled by lam^r and dKV scaled by lam^(Bk-r).
    `lambda_from_zero` swaps in the other printed variant of the row scale, lam^(r-1)."""
    n, d = Q.shape
    pos = np.arange(n, dtype=np.float64)
    r = np.arange(1, Bk + 1, dtype=np.float64)
    up = lam ** (r - 1 if lambda_from_zero else r)
    down = lam ** (Bk - r)
    O, dQ, dK, dV = (np.zeros_like(Q) for _ in range(4))
    for t0 in range(0, n, Bk):
        t1 = t0 + Bk
        blk = slice(t0, t1)
        q, k, v, g = (x[None, None, blk] for x in (Q, K, V, dO))
        O_in = oracle.left_product_fwd(q, k, v, [lam])[0, 0]
        dQ_in, dK_in, dV_in = (x[0, 0] for x in oracle.left_product_bwd(q, k, v, [lam], g))
        KV = np.einsum("s,si,sj->ij", lam ** (t0 - 1 - pos[:t0]), K[:t0], V[:t0])
        dKV = np.einsum("s,si,sj->ij", lam ** (pos[t1:] - t1 + 1), Q[t1:], dO[t1:])
        O[blk] = O_in + up[:, None] * (Q[blk] @ KV)
        dQ[blk] = dQ_in + up[:, None] * (dO[blk] @ KV.T)
        dK[blk] = dK_in + down[:, None] * (V[blk] @ dKV.T)
        dV[blk] = dV_in + down[:, None] * (K[blk] @ dKV)
    return O, dQ, dK, dV


@pytest.mark.parametrize("Bk", [1, 2, 4, 16])
@pytest.mark.parametrize("lam", [1.0, 0.9, 0.3])
def test_block_form_equals_token_form(Bk, lam):
    n, d = 16, 4
    Q, K, V, dO = _rand(1, 1, n, d, seed=31)
    ref = [oracle.c_recurrence_fwd(Q, K, V, [lam])[0, 0]] + \
        [x[0, 0] for x in oracle.c_recurrence_bwd(Q, K, V, [lam], dO)]
    for x, want in zip(_block_identities(Q[0, 0], K[0, 0], V[0, 0], lam, dO[0, 0], Bk), ref):
        np.testing.assert_allclose(x, want, rtol=1e-11, atol=1e-12)


def test_block_form_rejects_misprint():
    """With the proof's Lambda = diag(1, .., lam^(Bk-1)) the block form no
    longer matches the token form: the algorithm box's diag(lam, .., lam^Bk)
    is the reading to take."""
    n, d, Bk, lam = 16, 4, 4, 0.9
    Q, K, V, dO = _rand(1, 1, n, d, seed=33)
    ref = oracle.recurrence_fwd(Q, K, V, [lam])[0, 0]
    O, dQ, _, _ = _block_identities(Q[0, 0], K[0, 0], V[0, 0], lam, dO[0, 0], Bk, lambda_from_zero=True)
    assert np.max(np.abs(O - ref)) > 1e-2
    assert np.max(np.abs(dQ - oracle.recurrence_bwd(Q, K, V, [lam], dO)[0][0, 0])) > 1e-2


# ---- 8. causality --------------------------------------------------------------
@pytest.mark.parametrize("impl", list(FWD_IMPLS))
def test_causality(impl):
    n, d, s = 10, 3, 6
    Q, K, V, dO = _rand(1, 1, n, d, seed=41)
    O0 = FWD_IMPLS[impl](Q, K, V, [0.8])
    K2, V2 = K.copy(), V.copy()
    K2[0, 0, s] += 1.0
    V2[0, 0, s] -= 2.0
    O1 = FWD_IMPLS[impl](Q, K2, V2, [0.8])
    assert np.array_equal(O0[0, 0, :s], O1[0, 0, :s])
    assert np.all(np.any(O0[0, 0, s:] != O1[0, 0, s:], axis=1))
    g0 = BWD_IMPLS[impl](Q, K, V, [0.8], dO)
    dO2 = dO.copy()
    dO2[0, 0, s] += 1.0
    g1 = BWD_IMPLS[impl](Q, K, V, [0.8], dO2)
    for a, b in zip(g0[1:], g1[1:]):        # dK, dV change only at rows <= s
        assert np.array_equal(a[0, 0, s + 1:], b[0, 0, s + 1:])


# ---- 9. planted mistakes are caught (mistakes planted in a copy, on the CPU) ---
def test_planted_transposed_state_fails_example_b():
    g = load_golden("worked_example_b.txt")
    Q, K, V = g["Q"][0, 0], g["K"][0, 0], g["V"][0, 0]
    kv = np.zeros((2, 2))
    O = np.zeros((2, 2))
    for t in range(2):
        kv = g["lambda"] * kv + np.outer(V[t], K[t])      # wrong: v k^T
        O[t] = Q[t] @ kv
    assert np.max(np.abs(O - g["O"][0, 0])) > 0.5


def test_planted_exclusive_diagonal_fails_example_a():
    g = load_golden("worked_example_a.txt")
    Q, K, V = g["Q"][0, 0], g["K"][0, 0], g["V"][0, 0]
    kv = np.zeros((1, 1))
    O = np.zeros((3, 1))
    for t in range(3):
        O[t] = Q[t] @ kv                                    # wrong: state before update
        kv = g["lambda"] * kv + np.outer(K[t], V[t])
    assert np.max(np.abs(O - g["O"][0, 0])) > 0.5


# ---- 10. carried state: prefill in pieces and token-by-token decode -----------------
@pytest.mark.parametrize("lam", [1.0, 0.9, 0.2])
def test_state_carry_splits_the_sequence(lam):
    """Running the first m tokens, keeping kv_m, and continuing from it gives
    the same outputs as one run (the block form of App. C with blocks m, n-m),
    and the returned state is sum_s lam^(n-s) k_s v_s^T (App. C, KV_t)."""
    n, d, m = 13, 3, 5
    Q, K, V, _ = _rand(1, 1, n, d, seed=51)
    O_all = oracle.left_product_fwd(Q, K, V, [lam])
    O1, kv_m = oracle.recurrence_fwd(Q[:, :, :m], K[:, :, :m], V[:, :, :m], [lam], return_state=True)
    O2, kv_n = oracle.recurrence_fwd(Q[:, :, m:], K[:, :, m:], V[:, :, m:], [lam], kv0=kv_m,
                                     return_state=True)
    np.testing.assert_allclose(np.concatenate([O1, O2], axis=2), O_all, rtol=1e-11, atol=1e-12)
    w = lam ** (n - 1 - np.arange(n, dtype=np.float64))
    expect = (K[0, 0] * w[:, None]).T @ V[0, 0]
    np.testing.assert_allclose(kv_n[0, 0], expect, rtol=1e-11, atol=1e-12)


def test_decode_steps_reproduce_the_sequence():
    n, d, lam = 9, 4, [0.8, 1.0]
    Q, K, V, _ = _rand(2, 2, n, d, seed=52)
    O_all = oracle.left_product_fwd(Q, K, V, lam)
    kv = np.zeros((2, 2, d, d))
    for t in range(n):
        o, kv = oracle.decode_step(Q[:, :, t], K[:, :, t], V[:, :, t], lam, kv)
        np.testing.assert_allclose(o, O_all[:, :, t], rtol=1e-11, atol=1e-12)
    # worked example A: the state after the three tokens is 7.25
    g = load_golden("worked_example_a.txt")
    _, kv3 = oracle.recurrence_fwd(g["Q"], g["K"], g["V"], [g["lambda"]], return_state=True)
    assert abs(kv3[0, 0, 0, 0] - 7.25) < 1e-14


# ---- 11. gated SRMSNorm output stage (Sec. 4.2) --------------------------------------
def test_srmsnorm_worked_value_and_invariants():
    # x = (3, 4), D = 2: ||x|| = 5, x / (5 / sqrt 2) = (3, 4) * sqrt(2) / 5
    O = np.array([3.0, 4.0]).reshape(1, 1, 1, 2)
    U = np.ones_like(O)
    Y = oracle.gate_norm_fwd(O, U)
    np.testing.assert_allclose(Y.ravel(), np.array([3.0, 4.0]) * np.sqrt(2.0) / 5.0, rtol=1e-15)
    # heads are concatenated before the norm: two heads of one feature each give the same
    Y2 = oracle.gate_norm_fwd(O.reshape(1, 2, 1, 1), np.ones((1, 2, 1, 1)))
    np.testing.assert_allclose(Y2.ravel(), Y.ravel(), rtol=1e-15)
    rng = np.random.default_rng(3)
    O = rng.standard_normal((2, 3, 5, 4))
    U = rng.standard_normal((2, 3, 5, 4))
    N = oracle.gate_norm_fwd(O, np.ones_like(O))
    np.testing.assert_allclose(np.mean(N * N, axis=(1, 3)), 1.0, rtol=1e-12)       # unit mean square
    np.testing.assert_allclose(oracle.gate_norm_fwd(7.5 * O, U), oracle.gate_norm_fwd(O, U), rtol=1e-12)
    np.testing.assert_allclose(oracle.gate_norm_fwd(O, U), N * U, rtol=1e-12)      # the gate is a plain product


@pytest.mark.parametrize("eps", [0.0, 1e-3])
def test_gate_norm_gradients_by_finite_differences(eps):
    rng = np.random.default_rng(4)
    O = rng.standard_normal((1, 2, 3, 4))
    U = rng.standard_normal((1, 2, 3, 4))
    dY = rng.standard_normal((1, 2, 3, 4))
    dO, dU = oracle.gate_norm_bwd(O, U, dY, eps)
    h = 1e-6
    for which, grad in ((0, dO), (1, dU)):
        for idx in np.ndindex(O.shape):
            a = [O.copy(), U.copy()]
            b = [O.copy(), U.copy()]
            a[which][idx] += h
            b[which][idx] -= h
            fd = (np.sum(dY * oracle.gate_norm_fwd(a[0], a[1], eps)) -
                  np.sum(dY * oracle.gate_norm_fwd(b[0], b[1], eps))) / (2 * h)
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx]))
    if eps == 0.0:
        # the normalised output does not change along O: <dO, O> = 0 per token
        np.testing.assert_allclose(np.sum(dO * O, axis=(1, 3)), 0.0, atol=1e-12)


# ---- 12. Swish on the query / key projections (Sec. 4.2) ------------------------------
def test_swish_known_values_and_identities():
    # phi(0) = 0, phi'(0) = 1/2, phi(1) = 1 / (1 + 1/e), phi(-1) = -1 / (1 + e)
    assert oracle.swish(0.0) == 0.0
    assert oracle.swish_grad(0.0) == 0.5
    assert abs(oracle.swish(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16
    assert abs(oracle.swish(-1.0) + 1.0 / (1.0 + math.e)) < 1e-16
    # sigmoid(x) + sigmoid(-x) = 1  =>  phi(x) - phi(-x) = x  and  phi'(x) + phi'(-x) = 1
    x = np.linspace(-12.0, 12.0, 97)
    np.testing.assert_allclose(oracle.swish(x) - oracle.swish(-x), x, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.swish_grad(x) + oracle.swish_grad(-x), 1.0, rtol=0, atol=1e-14)
    # large |x|: phi -> x (right), -> 0 (left)
    assert abs(oracle.swish(40.0) - 40.0) < 1e-15 and abs(oracle.swish(-40.0)) < 1e-15
    # the single minimum: phi'(x*) = 0 gives x* sigma(x*) = 1 + x*, i.e. phi(x*) = 1 + x*;
    # found here by bisection on phi' alone
    lo, hi = -2.0, -1.0
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if oracle.swish_grad(mid) < 0.0:
            lo = mid
        else:
            hi = mid
    xs = 0.5 * (lo + hi)
    assert abs(xs + 1.2784645427610738) < 1e-12
    assert abs(oracle.swish(xs) - (1.0 + xs)) < 1e-12
    assert np.all(oracle.swish(x) >= oracle.swish(xs) - 1e-15)
    # derivative by central differences
    h = 1e-6
    fd = (oracle.swish(x + h) - oracle.swish(x - h)) / (2 * h)
    np.testing.assert_allclose(oracle.swish_grad(x), fd, rtol=0, atol=1e-8)


def test_swish_attention_gradients_by_finite_differences():
    """The composed loss <dO, attention(phi(Qp), phi(Kp), V)> differentiated
    numerically with respect to the pre-activations."""
    rng = np.random.default_rng(12)
    shape = (1, 2, 5, 3)
    lam = [0.8, 1.0]
    Qp, Kp, V, dO = (rng.standard_normal(shape) for _ in range(4))
    dQp, dKp, dV = oracle.swish_attention_bwd(Qp, Kp, V, lam, dO)
    loss = lambda q, k, v: float(np.sum(dO * oracle.left_product_fwd(oracle.swish(q), oracle.swish(k), v, lam)))
    h = 1e-6
    for which, grad in ((0, dQp), (1, dKp), (2, dV)):
        for idx in np.ndindex(shape):
            a = [Qp.copy(), Kp.copy(), V.copy()]
            b = [Qp.copy(), Kp.copy(), V.copy()]
            a[which][idx] += h
            b[which][idx] -= h
            fd = (loss(*a) - loss(*b)) / (2 * h)
            assert abs(fd - grad[idx]) <= 2e-8 * max(1.0, abs(grad[idx])), (which, idx)
    # forward: the activation is applied to Q and K only, never to V
    O = oracle.swish_attention_fwd(Qp, Kp, V, lam)
    np.testing.assert_allclose(O, oracle.left_product_fwd(oracle.swish(Qp), oracle.swish(Kp), V, lam), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(oracle.swish_attention_fwd(Qp, Kp, 2.0 * V, lam), 2.0 * O, rtol=1e-12)


# ---- 13. wider query / key features and LRPE-d (Sec. 4.1) ------------------------------
def test_wide_keys_are_a_sum_over_feature_slices():
    """With d_k = 2 d_v the scores add over the two halves of the features, so the
    attention (both forms) is the sum of two ordinary ones, and so is dV; dQ, dK split."""
    rng = np.random.default_rng(21)
    B, H, n, dv = 1, 2, 9, 3
    lam = [0.7, 1.0]
    Qw, Kw = rng.standard_normal((B, H, n, 2 * dv)), rng.standard_normal((B, H, n, 2 * dv))
    V, dO = rng.standard_normal((B, H, n, dv)), rng.standard_normal((B, H, n, dv))
    O = oracle.left_product_fwd(Qw, Kw, V, lam)
    np.testing.assert_allclose(O, oracle.recurrence_fwd(Qw, Kw, V, lam), rtol=1e-12, atol=1e-13)
    parts = [oracle.left_product_fwd(Qw[..., j * dv:(j + 1) * dv], Kw[..., j * dv:(j + 1) * dv], V, lam) for j in (0, 1)]
    np.testing.assert_allclose(O, parts[0] + parts[1], rtol=1e-12, atol=1e-13)
    dQw, dKw, dV = oracle.left_product_bwd(Qw, Kw, V, lam, dO)
    r = oracle.recurrence_bwd(Qw, Kw, V, lam, dO)
    for a, b in zip((dQw, dKw, dV), r):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    dv_sum = np.zeros_like(dV)
    for j in (0, 1):
        sl = slice(j * dv, (j + 1) * dv)
        g = oracle.left_product_bwd(Qw[..., sl], Kw[..., sl], V, lam, dO)
        np.testing.assert_allclose(dQw[..., sl], g[0], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(dKw[..., sl], g[1], rtol=1e-12, atol=1e-13)
        dv_sum += g[2]
    np.testing.assert_allclose(dV, dv_sum, rtol=1e-12, atol=1e-13)
    # finite differences of <dO, O> with respect to one entry of each wide operand
    h = 1e-6
    loss = lambda q, k, v: float(np.sum(dO * oracle.left_product_fwd(q, k, v, lam)))
    for which, grad in ((0, dQw), (1, dKw), (2, dV)):
        for idx in [(0, 0, 0, 0), (0, 1, 4, 2), (0, 1, n - 1, grad.shape[3] - 1)]:
            a = [Qw.copy(), Kw.copy(), V.copy()]
            b = [Qw.copy(), Kw.copy(), V.copy()]
            a[which][idx] += h
            b[which][idx] -= h
            assert abs((loss(*a) - loss(*b)) / (2 * h) - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx]))


def test_lrpe_definition_equals_attention_over_rotated_features():
    """The score q_t^T k_s lambda^(t-s) Re exp(i theta (t-s)), written out term by term,
    equals the ordinary (wide) attention over the cos / sin features."""
    rng = np.random.default_rng(22)
    B, H, n, d = 1, 2, 7, 3
    lam = [0.8, 1.0]
    theta = rng.uniform(0.0, 2.0, size=(H, d))
    Q, K, V = (rng.standard_normal((B, H, n, d)) for _ in range(3))
    O_def = oracle.lrpe_fwd(Q, K, V, lam, theta)
    Qw, Kw = oracle.lrpe_features(Q, theta), oracle.lrpe_features(K, theta)
    assert Qw.shape == (B, H, n, 2 * d)
    np.testing.assert_allclose(oracle.left_product_fwd(Qw, Kw, V, lam), O_def, rtol=1e-12, atol=1e-13)
    # theta = 0: no rotation, the plain attention
    zero = np.zeros((H, d))
    np.testing.assert_allclose(oracle.lrpe_fwd(Q, K, V, lam, zero), oracle.left_product_fwd(Q, K, V, lam),
                               rtol=1e-12, atol=1e-13)
    # one feature, constant q = k = v = 1, lambda = 1: O[t] = sum_{m=0..t} cos(m theta)  (Dirichlet kernel sum)
    th = 0.37
    one = np.ones((1, 1, 6, 1))
    O1 = oracle.lrpe_fwd(one, one, one, [1.0], np.array([[th]]))
    closed = np.array([np.sin((t + 1) * th / 2) * np.cos(t * th / 2) / np.sin(th / 2) for t in range(6)])
    np.testing.assert_allclose(O1.ravel(), closed, rtol=1e-12)
    # only differences of positions matter: dropping the first token of a sequence whose first
    # key/value row is zero leaves the later outputs unchanged
    K0, V0 = K.copy(), V.copy()
    K0[:, :, 0] = 0.0
    V0[:, :, 0] = 0.0
    full = oracle.lrpe_fwd(Q, K0, V0, lam, theta)
    cut = oracle.lrpe_fwd(Q[:, :, 1:], K0[:, :, 1:], V0[:, :, 1:], lam, theta)
    np.testing.assert_allclose(full[:, :, 1:], cut, rtol=1e-12, atol=1e-13)


def test_lrpe_feature_gradients_by_finite_differences():
    rng = np.random.default_rng(23)
    B, H, n, d = 2, 2, 6, 3
    theta = rng.uniform(0.0, 2.0, size=(H, d))
    X = rng.standard_normal((B, H, n, d))
    G = rng.standard_normal((B, H, n, 2 * d))
    dX, dtheta = oracle.lrpe_features_bwd(X, theta, G)
    loss = lambda x, th: float(np.sum(G * oracle.lrpe_features(x, th)))
    h = 1e-6
    for idx in np.ndindex(X.shape):
        a, b = X.copy(), X.copy()
        a[idx] += h
        b[idx] -= h
        assert abs((loss(a, theta) - loss(b, theta)) / (2 * h) - dX[idx]) <= 1e-8 * max(1.0, abs(dX[idx]))
    for idx in np.ndindex(theta.shape):
        a, b = theta.copy(), theta.copy()
        a[idx] += h
        b[idx] -= h
        assert abs((loss(X, a) - loss(X, b)) / (2 * h) - dtheta[idx]) <= 1e-7 * max(1.0, abs(dtheta[idx]))
    # rotation keeps the norm of every row pair: |Xw|^2 = |X|^2
    Xw = oracle.lrpe_features(X, theta)
    np.testing.assert_allclose(np.sum(Xw * Xw, axis=3), np.sum(X * X, axis=3), rtol=1e-12)
    # row 0 is not rotated
    np.testing.assert_allclose(Xw[:, :, 0, :d], X[:, :, 0])
    np.testing.assert_allclose(Xw[:, :, 0, d:], 0.0, atol=0)
