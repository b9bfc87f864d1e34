"""CPU oracle for causal linear attention with per-head decay (fp64, NumPy).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
GPU library must compute.  It shares no code with the HIP path, is never
imported by it, and is only used by the tests, the smoke check and the CPU
baseline leg of the benchmark.

Two independent forms of the same exact result are given, per (batch, head):

  form (i)  "left product" (Alg. 1, Eq. 3 of Sec. 3.1, with the decay mask of
            App. A, first equation block):
                A[t, s] = lambda^(t-s) if t >= s else 0          (diagonal = 1)
                P = (Q K^T) * A ,   O = P V
            and its gradients, with G = (dO V^T) * A:
                dQ = G K ,  dK = G^T Q ,  dV = P^T dO
            (the n-row statement of the intra-block lines of Alg. 6).

  form (ii) "right product" recurrence (Alg. 2; with decay: App. A second
            equation block and App. C "Forward Pass"/"Backward Pass"):
                kv_0 = 0,  kv_t = lambda kv_{t-1} + k_t v_t^T,  o_t^T = q_t^T kv_t
                dq_t^T = do_t^T kv_t^T
                dkv_{n+1} = 0,  dkv_t = lambda dkv_{t+1} + q_t do_t^T
                dk_t^T = v_t^T dkv_t^T ,  dv_t^T = k_t^T dkv_t
            kv_t and dkv_t are d x d with rows = key feature, cols = value
            feature.  dkv_t includes the term of position t itself.

Readings taken where the paper's text is inconsistent:
  * the mask diagonal is included (a token attends to itself), as Alg. 1 and
    Alg. 5 state and as o_t = q_t^T kv_t with kv_t containing k_t v_t^T implies;
  * outer products are always k v^T (d x d), whatever row/column notation a
    given line of the appendix uses;
  * lambda is a constant: no gradient flows to it (Sec. 4.1 keeps it fixed);
  * no 1/sqrt(d) scaling and no normalisation are applied (Sec. 3.1).

All arithmetic is fp64.  Tensors are [B, H, n, d]; `lam` has H entries.
"""
from __future__ import annotations

import numpy as np


def _as64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def decay_matrix(n: int, lam: float) -> np.ndarray:
    """A[t, s] = lam^(t-s) for t >= s, else 0 (n x n, fp64)."""
    t = np.arange(n)[:, None]
    s = np.arange(n)[None, :]
    diff = t - s
    A = np.zeros((n, n), dtype=np.float64)
    mask = diff >= 0
    A[mask] = np.power(float(lam), diff[mask].astype(np.float64))
    return A


# --------------------------------------------------------------------------
# form (i): quadratic masked form
# --------------------------------------------------------------------------
def left_product_fwd(Q, K, V, lam):
    """Q, K: [B, H, n, d_k]; V: [B, H, n, d_v] (d_k = d_v in the paper's layers; a wider
    query / key feature, as the cos / sin features of LRPE-d give, changes nothing here)."""
    Q, K, V = _as64(Q), _as64(K), _as64(V)
    B, H, n, d = Q.shape
    O = np.empty_like(V)
    for h in range(H):
        A = decay_matrix(n, lam[h])
        for b in range(B):
            P = (Q[b, h] @ K[b, h].T) * A
            O[b, h] = P @ V[b, h]
    return O


def left_product_bwd(Q, K, V, lam, dO):
    Q, K, V, dO = _as64(Q), _as64(K), _as64(V), _as64(dO)
    B, H, n, d = Q.shape
    dQ = np.empty_like(Q)
    dK = np.empty_like(K)
    dV = np.empty_like(V)
    for h in range(H):
        A = decay_matrix(n, lam[h])
        for b in range(B):
            P = (Q[b, h] @ K[b, h].T) * A
            G = (dO[b, h] @ V[b, h].T) * A
            dQ[b, h] = G @ K[b, h]
            dK[b, h] = G.T @ Q[b, h]
            dV[b, h] = P.T @ dO[b, h]
    return dQ, dK, dV


# --------------------------------------------------------------------------
# form (ii): token-by-token recurrence
# --------------------------------------------------------------------------
def recurrence_fwd(Q, K, V, lam, kv0=None, return_state=False):
    """Token recurrence.  With `kv0` ([B, H, d, d]) the recurrence starts from
    that state instead of zero (the state left by earlier tokens: Sec. 3.1 notes
    that inference only ever needs this d x d state); with `return_state` the
    state after the last token, kv_n, is returned as well."""
    Q, K, V = _as64(Q), _as64(K), _as64(V)
    B, H, n, d = Q.shape
    dv = V.shape[3]
    O = np.empty_like(V)
    KVn = np.empty((B, H, d, dv), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            l = float(lam[h])
            kv = np.zeros((d, dv), dtype=np.float64) if kv0 is None else _as64(kv0)[b, h].copy()
            for t in range(n):
                kv = l * kv + np.outer(K[b, h, t], V[b, h, t])
                O[b, h, t] = Q[b, h, t] @ kv
            KVn[b, h] = kv
    return (O, KVn) if return_state else O


def decode_step(q, k, v, lam, kv):
    """One token of the recurrence (App. A, recurrence form): kv' = lam kv + k v^T,
    o = q^T kv'.  q, k, v: [B, H, d]; kv: [B, H, d, d].  Returns (o, kv')."""
    q, k, v, kv = _as64(q), _as64(k), _as64(v), _as64(kv)
    B, H, d = q.shape
    o = np.empty_like(q)
    kv_new = np.empty_like(kv)
    for b in range(B):
        for h in range(H):
            kv_new[b, h] = float(lam[h]) * kv[b, h] + np.outer(k[b, h], v[b, h])
            o[b, h] = q[b, h] @ kv_new[b, h]
    return o, kv_new


def recurrence_bwd(Q, K, V, lam, dO):
    Q, K, V, dO = _as64(Q), _as64(K), _as64(V), _as64(dO)
    B, H, n, d = Q.shape
    dv = V.shape[3]
    dQ = np.empty_like(Q)
    dK = np.empty_like(K)
    dV = np.empty_like(V)
    for b in range(B):
        for h in range(H):
            l = float(lam[h])
            kv = np.zeros((d, dv), dtype=np.float64)
            for t in range(n):
                kv = l * kv + np.outer(K[b, h, t], V[b, h, t])
                dQ[b, h, t] = kv @ dO[b, h, t]
            dkv = np.zeros((d, dv), dtype=np.float64)
            for t in range(n - 1, -1, -1):
                dkv = l * dkv + np.outer(Q[b, h, t], dO[b, h, t])
                dK[b, h, t] = dkv @ V[b, h, t]
                dV[b, h, t] = K[b, h, t] @ dkv
    return dQ, dK, dV


def rel_max_err(x, ref) -> float:
    """max|x - ref| / max|ref| over the whole tensor (the error measure the
    parity tolerances are stated in)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(x)))
    return float(np.max(np.abs(x - ref)) / denom)


# --------------------------------------------------------------------------
# gated, normalised output of the attention block (Sec. 4.2, "Gating Mechanism"
# and "Tensor Normalization"): Y = SRMSNorm(O) * U, SRMSNorm(x) = x / (||x||_2 / sqrt(D))
# --------------------------------------------------------------------------
def gate_norm_fwd(O, U, eps=0.0):
    """O, U: [B, H, n, d].  The norm runs per token over all H*d features of
    the attention output (the heads concatenated).  `eps` is added to the mean
    square before the root; the paper's formula is eps = 0."""
    O, U = _as64(O), _as64(U)
    B, H, n, d = O.shape
    ms = np.mean(O * O, axis=(1, 3), keepdims=True) + eps      # [B,1,n,1]
    return O / np.sqrt(ms) * U


def gate_norm_bwd(O, U, dY, eps=0.0):
    """Gradients of Y = SRMSNorm(O) * U:  with r = sqrt(mean(O^2)+eps), N = O/r,
    dN = dY*U:  dU = dY*N,  dO = dN/r - O * mean(dN*O) / r^3."""
    O, U, dY = _as64(O), _as64(U), _as64(dY)
    ms = np.mean(O * O, axis=(1, 3), keepdims=True) + eps
    r = np.sqrt(ms)
    dN = dY * U
    dU = dY * O / r
    c = np.mean(dN * O, axis=(1, 3), keepdims=True)
    dO = dN / r - O * c / (r ** 3)
    return dO, dU


# --------------------------------------------------------------------------
# activation of the query / key projections (Sec. 4.2, "Gating Mechanism":
# Q = phi(X W_q), K = phi(X W_k), phi = Swish).  Reading: Swish with beta = 1,
# phi(x) = x * sigmoid(x); the paper names the function and gives no beta.
# --------------------------------------------------------------------------
def swish(x):
    """phi(x) = x / (1 + exp(-x)), fp64."""
    x = _as64(x)
    with np.errstate(over="ignore"):        # exp(-x) = inf for x << 0 gives the limit 0
        return x / (1.0 + np.exp(-x))


def swish_grad(x):
    """phi'(x) = s + x s (1 - s), s = sigmoid(x)."""
    x = _as64(x)
    with np.errstate(over="ignore"):
        s = 1.0 / (1.0 + np.exp(-x))
    return s + x * s * (1.0 - s)


def swish_attention_fwd(Qp, Kp, V, lam):
    """O = attention(phi(Qp), phi(Kp), V): the attention of this file applied
    to the activated projections."""
    return recurrence_fwd(swish(Qp), swish(Kp), V, lam)


def swish_attention_bwd(Qp, Kp, V, lam, dO):
    """Gradients with respect to the pre-activations: chain rule through phi,
    dQp = dQ * phi'(Qp), dKp = dK * phi'(Kp); dV is the attention's own."""
    dQ, dK, dV = recurrence_bwd(swish(Qp), swish(Kp), V, lam, dO)
    return dQ * swish_grad(Qp), dK * swish_grad(Kp), dV


# --------------------------------------------------------------------------
# LRPE-d (Sec. 4.1, "Position Encoding"):  a_ts = q_t^T k_s lambda^(t-s) exp(i theta (t-s)).
# Readings: theta is one angle per head and feature ([H, d]); the attention score is the
# real part,  sum_i q_ti k_si cos(theta_i (t - s));  positions count from 0 (only the
# differences t - s enter).
# --------------------------------------------------------------------------
def lrpe_fwd(Q, K, V, lam, theta):
    """The definition written out: O[t] = sum_{s<=t} lambda^(t-s) [sum_i q_ti k_si cos(theta_i (t-s))] v_s."""
    Q, K, V, theta = _as64(Q), _as64(K), _as64(V), _as64(theta)
    B, H, n, d = Q.shape
    O = np.zeros_like(V)
    for b in range(B):
        for h in range(H):
            for t in range(n):
                for s in range(t + 1):
                    score = np.sum(Q[b, h, t] * K[b, h, s] * np.cos(theta[h] * (t - s)))
                    O[b, h, t] += float(lam[h]) ** (t - s) * score * V[b, h, s]
    return O


def lrpe_features(X, theta):
    """The decomposition the paper points to ("can be decomposed with respect to s and t
    separately"): x_t -> [x_t cos(t theta), x_t sin(t theta)], so that the plain inner
    product of two feature rows is sum_i x_ti y_si cos(theta_i (t - s))."""
    X, theta = _as64(X), _as64(theta)
    B, H, n, d = X.shape
    ang = np.arange(n, dtype=np.float64)[None, :, None] * theta[:, None, :]      # [H, n, d]
    return np.concatenate([X * np.cos(ang)[None], X * np.sin(ang)[None]], axis=3)


def lrpe_features_bwd(X, theta, dXw):
    """Gradients of Xw = lrpe_features(X, theta) given dXw ([B, H, n, 2d]):
    dX = dXw_c cos(t theta) + dXw_s sin(t theta);
    dtheta[h, i] = sum_{b, t} t x_ti (dXw_s cos(t theta_i) - dXw_c sin(t theta_i))."""
    X, theta, dXw = _as64(X), _as64(theta), _as64(dXw)
    B, H, n, d = X.shape
    t = np.arange(n, dtype=np.float64)[None, :, None]
    ang = t * theta[:, None, :]                                   # [H, n, d]
    c, s = np.cos(ang)[None], np.sin(ang)[None]
    gc, gs = dXw[..., :d], dXw[..., d:]
    dX = gc * c + gs * s
    dtheta = np.sum(t[None] * X * (gs * c - gc * s), axis=(0, 2))
    return dX, dtheta
