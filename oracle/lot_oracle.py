"""ctypes front end of the CPU oracle in lot_oracle.c (test infrastructure, not the product).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this module.  It
holds no arithmetic of its own apart from the marginal residuals at the end, which are the
plain definitions (row and column sums compared with the prescribed masses).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lot_oracle.c")
_LIB = os.path.join(_HERE, "liblot_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile lot_oracle.c with gcc (OpenMP over the independent problems only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.lot_oracle_attention.restype = ctypes.c_int
    return _lib


def _d(x):
    a = np.ascontiguousarray(x, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def cost(X, Z):
    """C = X Z^T  (n x r)."""
    X, px = _d(X)
    Z, pz = _d(Z)
    n, d = X.shape
    r = Z.shape[0]
    C = np.empty((n, r), dtype=np.float64)
    _load().lot_oracle_cost(px, pz, n, r, d, C.ctypes.data_as(_dp))
    return C


def sinkhorn(C, a, b, eps, T):
    """Potentials (f, g) after T iterations started from g = 0."""
    C, pc = _d(C)
    a, pa = _d(a)
    b, pb = _d(b)
    n, r = C.shape
    f = np.empty(n, dtype=np.float64)
    g = np.empty(r, dtype=np.float64)
    _load().lot_oracle_sinkhorn(pc, n, r, pa, pb, ctypes.c_double(eps), int(T),
                                f.ctypes.data_as(_dp), g.ctypes.data_as(_dp))
    return f, g


def coupling(C, f, g, eps):
    C, pc = _d(C)
    f, pf = _d(f)
    g, pg = _d(g)
    n, r = C.shape
    G = np.empty((n, r), dtype=np.float64)
    _load().lot_oracle_coupling(pc, pf, pg, n, r, ctypes.c_double(eps), G.ctypes.data_as(_dp))
    return G


def couplings_one(Q, K, Z, beta, eps, T):
    """gamma1 (n x r), gamma2 (r x n) of one problem."""
    Q, pq = _d(Q)
    K, pk = _d(K)
    Z, pz = _d(Z)
    beta, pb = _d(beta)
    n, d = Q.shape
    r = Z.shape[0]
    g1 = np.empty((n, r), dtype=np.float64)
    g2 = np.empty((r, n), dtype=np.float64)
    _load().lot_oracle_couplings_one(pq, pk, pz, pb, n, d, r, ctypes.c_double(eps), int(T),
                                     g1.ctypes.data_as(_dp), g2.ctypes.data_as(_dp))
    return g1, g2


def apply_factored(gamma1, gamma2, beta, V):
    g1, p1 = _d(gamma1)
    g2, p2 = _d(gamma2)
    beta, pb = _d(beta)
    V, pv = _d(V)
    n, r = g1.shape
    d_v = V.shape[1]
    O = np.empty((n, d_v), dtype=np.float64)
    _load().lot_oracle_apply_factored(p1, p2, pb, pv, n, r, d_v, O.ctypes.data_as(_dp))
    return O


def dense_plan(gamma1, gamma2, beta):
    g1, p1 = _d(gamma1)
    g2, p2 = _d(gamma2)
    beta, pb = _d(beta)
    n, r = g1.shape
    P = np.empty((n, n), dtype=np.float64)
    _load().lot_oracle_dense_plan(p1, p2, pb, n, r, P.ctypes.data_as(_dp))
    return P


def outer_plan(gamma1, gamma2, beta):
    g1, p1 = _d(gamma1)
    g2, p2 = _d(gamma2)
    beta, pb = _d(beta)
    n, r = g1.shape
    P = np.empty((n, n), dtype=np.float64)
    _load().lot_oracle_outer_plan(p1, p2, pb, n, r, P.ctypes.data_as(_dp))
    return P


def apply_dense(P, V):
    P, pp = _d(P)
    V, pv = _d(V)
    n = P.shape[0]
    d_v = V.shape[1]
    O = np.empty((n, d_v), dtype=np.float64)
    _load().lot_oracle_apply_dense(pp, pv, n, d_v, O.ctypes.data_as(_dp))
    return O


def attention(Q, K, V, Z, beta, eps, T, want_couplings=False, threads=1):
    """O [B,H,n,d_v] (and gamma1 [B,H,n,r], gamma2 [B,H,r,n]) for a whole batch."""
    Q, pq = _d(Q)
    K, pk = _d(K)
    V, pv = _d(V)
    Z, pz = _d(Z)
    beta, pb = _d(beta)
    B, H, n, d_k = Q.shape
    d_v = V.shape[3]
    r = Z.shape[1]
    O = np.empty((B, H, n, d_v), dtype=np.float64)
    if want_couplings:
        g1 = np.empty((B, H, n, r), dtype=np.float64)
        g2 = np.empty((B, H, r, n), dtype=np.float64)
        p1, p2 = g1.ctypes.data_as(_dp), g2.ctypes.data_as(_dp)
    else:
        g1 = g2 = None
        p1 = p2 = _dp()
    used = _load().lot_oracle_attention(B, H, n, d_k, d_v, r, pq, pk, pv, pz, pb,
                                        ctypes.c_double(eps), int(T),
                                        O.ctypes.data_as(_dp), p1, p2, int(threads))
    if want_couplings:
        return O, g1, g2, used
    return O, used


def marginal_residuals(gamma1, gamma2, beta):
    """The four residual vectors of the couplings' marginals (uniform token masses 1/n).

    tok1_i = n sum_t gamma1[i,t] - 1,  piv1_t = sum_i gamma1[i,t] / beta_t - 1,
    tok2_j = n sum_t gamma2[t,j] - 1,  piv2_t = sum_j gamma2[t,j] / beta_t - 1.
    Leading batch dimensions are allowed; beta broadcasts over them.
    """
    g1 = np.asarray(gamma1, dtype=np.float64)
    g2 = np.asarray(gamma2, dtype=np.float64)
    b = np.asarray(beta, dtype=np.float64)
    n = g1.shape[-2]
    tok1 = n * g1.sum(axis=-1) - 1.0
    piv1 = g1.sum(axis=-2) / b - 1.0
    tok2 = n * g2.sum(axis=-2) - 1.0
    piv2 = g2.sum(axis=-1) / b - 1.0
    return tok1, piv1, tok2, piv2


def attention_cls(Q, K, V, Z, beta, eps, T, beta_cls, threads=1):
    """ViT variant with a [CLS] token at index 0 (paper, "[CLS] under DS attention").

    Rows 1..n-1: the doubly-stochastic LOT attention among tokens 1..n-1 only (their own queries,
    keys and values; masses 1/(n-1)), i.e. `attention` on the views without token 0.  Row 0: a
    standard softmax row over ALL n keys with temperature beta_cls,
    alpha_j = exp(beta_cls <q_0, k_j>) / sum_l exp(beta_cls <q_0, k_l>), out_0 = sum_j alpha_j v_j,
    written out below with the usual maximum subtraction.  The paper does not say how [CLS] enters as
    a key of the other rows; the reading taken is the literal one ("DS constraints only among the
    image tokens"): it does not.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, n, _ = Q.shape
    out = np.empty(V.shape, dtype=np.float64)
    inner, _ = attention(Q[:, :, 1:], K[:, :, 1:], V[:, :, 1:], Z, beta, eps, T, threads=threads)
    out[:, :, 1:] = inner
    for b in range(B):
        for h in range(H):
            score = np.array([beta_cls * float(np.dot(Q[b, h, 0], K[b, h, j])) for j in range(n)])
            w = np.exp(score - score.max())
            w /= w.sum()
            acc = np.zeros(V.shape[-1])
            for j in range(n):
                acc += w[j] * V[b, h, j]
            out[b, h, 0] = acc
    return out


def cross_attention(Q, K, V, Z, beta, mass_q, mass_k, eps, T):
    """Cross attention / non-uniform token masses (paper, "Empirical measures and pivot": mu = sum_i
    p1_i delta_{q_i}, nu = sum_j p2_j delta_{k_j}; "Glued coupling": Gamma 1 = mu, Gamma^T 1 = nu).

    Q [B,H,n_q,d_k], K [B,H,n_k,d_k], V [B,H,n_k,d_v], mass_q [B,H,n_q], mass_k [B,H,n_k]: nonnegative,
    each summing to one; a token of mass zero is padding.  Per problem: C1 = Q Z^T, C2 = K Z^T; the two
    Sinkhorn solves with marginals (mass_q, beta) and (mass_k, beta), token side first, pivot side
    last, T iterations from g = 0; Gamma2 = exp((C2 + f2 + g2)/eps); Y' = Diag(beta)^-1 Gamma2^T V;
    and the attention is the glued plan with its rows renormalised, A = Diag(mu)^-1 Gamma, which is
    what A = n Gamma is for uniform masses (reading: the paper writes A only for the balanced case).
    Row i of Diag(mu)^-1 Gamma1 is exp((C1_it + g1_t)/eps) / sum_t' exp((C1_it' + g1prev_t')/eps) with
    g1prev the pivot potentials before the last pivot-side update -- the token potential
    f_i = eps (log mu_i - LSE) cancels mu_i -- so it is defined for zero-mass queries as well.
    Returns O [B,H,n_q,d_v].
    """
    Q = np.asarray(Q, dtype=np.float64); K = np.asarray(K, dtype=np.float64); V = np.asarray(V, dtype=np.float64)
    B, H, n_q, _ = Q.shape
    out = np.empty((B, H, n_q, V.shape[-1]), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            bt = np.asarray(beta[h], dtype=np.float64)
            C1 = cost(Q[b, h], Z[h])
            C2 = cost(K[b, h], Z[h])
            with np.errstate(divide="ignore"):
                _, g1 = sinkhorn(C1, mass_q[b, h], bt, eps, T)
                _, g1prev = sinkhorn(C1, mass_q[b, h], bt, eps, T - 1) if T > 1 else (None, np.zeros_like(bt))
                f2, g2 = sinkhorn(C2, mass_k[b, h], bt, eps, T)
            gamma2 = coupling(C2, f2, g2, eps)                       # n_k x r, zero rows for zero masses
            Yp = (gamma2.T @ V[b, h]) / bt[:, None]
            x = (C1 + g1prev[None, :]) / eps
            m = x.max(axis=1, keepdims=True)
            lse = m + np.log(np.exp(x - m).sum(axis=1, keepdims=True))
            R1 = np.exp((C1 + g1[None, :]) / eps - lse)               # rows of Diag(mu)^-1 Gamma1
            out[b, h] = R1 @ Yp
    return out
