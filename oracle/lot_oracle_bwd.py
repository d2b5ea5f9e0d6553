"""CPU oracle of the LOT attention BACKWARD pass (test infrastructure, not the product).

The paper trains the pivots, their masses and the projections by backpropagating through the two
Sinkhorn problems and the glued composition ("Learning" paragraph), with ordinary automatic
differentiation of an unfused implementation (FlashAttention-comparison appendix).  The gradient of
a finite number of Sinkhorn iterations has a plain definition -- the derivative of the forward
function -- so this oracle IS that definition: the forward pass written once more with plain PyTorch
CPU operations in float64, exactly in the order of the paper's algorithm

    C1 = Q Z^T, C2 = K Z^T                                   (similarity, "Computation" paragraph)
    g <- 0;  T x { f_i <- eps (log a_i - LSE_t((C_it + g_t)/eps)) ;
                   g_t <- eps (log b_t - LSE_i((C_it + f_i)/eps)) }          (Sinkhorn scaling form)
    Gamma_it = exp((C_it + f_i + g_t)/eps)
    O = n * Gamma1 Diag(beta)^-1 Gamma2 V                    (glued plan, factored apply)

and differentiated by torch.autograd.  Nothing is fused, blocked or reordered.

Pinned (tests/test_oracle_bwd_pins.py) by things that are not this file: its forward agrees with the
C oracle; its gradients agree with central finite differences OF THE C ORACLE's forward; closed
forms (one pivot: O = beta_1 mean(V), which fixes dV and dbeta and makes dQ, dK, dZ vanish; a common
shift of all pivots changes no coupling, so the pivot gradients of a head sum to zero; O is linear
in V, so dV = A^T dO with the dense plan A = n P built by the C oracle).

The [CLS] variant ("[CLS] under DS attention") is differentiated the same way: its forward (row 0 a
softmax row over all keys, rows 1.. the method among the other tokens) written with plain torch
operations, pinned by the numpy/C oracle of that variant, by its central finite differences, and by
the two cases in which one of the two parts receives no gradient.

Cross attention with token masses ("Empirical measures and pivot", "Glued coupling") likewise:
`forward_cross` is the two solves with marginals (mass_q, beta) and (mass_k, beta) and the glued
plan with renormalised rows, written with plain torch operations; the masses are data (a padding
mask), not differentiated.  Pinned by the numpy/C oracle of that forward, its central finite
differences, the uniform case (which is `forward`) and padding (zero-mass keys receive no gradient
and change nobody else's).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.
"""
from __future__ import annotations

import numpy as np
import torch


def _solve(C, a_log, b_log, eps, T):
    """Potentials after T iterations from g = 0; C is [..., n, r], b_log is [..., 1, r]."""
    g = torch.zeros_like(b_log)
    f = None
    for _ in range(T):
        f = eps * (a_log - torch.logsumexp((C + g) / eps, dim=-1, keepdim=True))      # [..., n, 1]
        g = eps * (b_log - torch.logsumexp((C + f) / eps, dim=-2, keepdim=True))      # [..., 1, r]
    return f, g


def forward(Q, K, V, Z, beta, eps, T):
    """O[B,H,n,d_v] for torch float64 tensors Q,K [B,H,n,d_k], V [B,H,n,d_v], Z [H,r,d_k], beta [H,r]."""
    n = Q.shape[-2]
    a_log = torch.log(torch.tensor(1.0 / n, dtype=Q.dtype))
    b_log = torch.log(beta)[None, :, None, :]                                          # [1,H,1,r]
    C1 = torch.einsum("bhnc,hrc->bhnr", Q, Z)
    C2 = torch.einsum("bhnc,hrc->bhnr", K, Z)
    f1, g1 = _solve(C1, a_log, b_log, eps, T)
    f2, g2 = _solve(C2, a_log, b_log, eps, T)
    gamma1 = torch.exp((C1 + f1 + g1) / eps)                                           # [B,H,n,r]
    gamma2 = torch.exp((C2 + f2 + g2) / eps)                                           # [B,H,n,r] (transposed plan)
    Y = torch.einsum("bhnr,bhnc->bhrc", gamma2, V)                                     # Gamma2 V
    Yp = Y / beta[None, :, :, None]
    return n * torch.einsum("bhnr,bhrc->bhnc", gamma1, Yp)


def attention_bwd(Q, K, V, Z, beta, eps, T, dO):
    """Gradients of <O, dO> with respect to Q, K, V, Z, beta (numpy float64 in and out).

    Z and beta are per head and shared over the batch, so their gradients are summed over it.
    """
    t = [torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True) for x in (Q, K, V, Z, beta)]
    O = forward(*t, float(eps), int(T))
    loss = (O * torch.tensor(np.asarray(dO, dtype=np.float64))).sum()
    grads = torch.autograd.grad(loss, t)
    return tuple(g.detach().numpy() for g in grads), O.detach().numpy()


def forward_cls(Q, K, V, Z, beta, eps, T, beta_cls):
    """[CLS] variant: row 0 = softmax_j(beta_cls[b,h] <q_0, k_j>) V over all n keys; rows 1..n-1 =
    `forward` on tokens 1..n-1.  beta_cls is a [B,H] tensor (one temperature per problem)."""
    inner = forward(Q[..., 1:, :], K[..., 1:, :], V[..., 1:, :], Z, beta, eps, T)
    score = beta_cls[..., None] * torch.einsum("bhc,bhnc->bhn", Q[..., 0, :], K)
    row0 = torch.einsum("bhn,bhnc->bhc", torch.softmax(score, dim=-1), V)
    return torch.cat([row0[..., None, :], inner], dim=-2)


def attention_cls_bwd(Q, K, V, Z, beta, eps, T, beta_cls, dO):
    """Gradients of <O, dO> for the [CLS] variant with respect to Q, K, V, Z, beta and, per (b, h)
    problem, the temperature (array [B,H]; its sum is the gradient of a shared scalar)."""
    t = [torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True) for x in (Q, K, V, Z, beta)]
    bc = torch.full(t[0].shape[:2], float(beta_cls), dtype=torch.float64, requires_grad=True)
    O = forward_cls(*t, float(eps), int(T), bc)
    loss = (O * torch.tensor(np.asarray(dO, dtype=np.float64))).sum()
    grads = torch.autograd.grad(loss, t + [bc])
    return tuple(g.detach().numpy() for g in grads), O.detach().numpy()


def forward_cross(Q, K, V, Z, beta, mass_q, mass_k, eps, T):
    """O[B,H,n_q,d_v] = Diag(mu)^-1 Gamma1 Diag(beta)^-1 Gamma2 V for Q [B,H,n_q,d_k], K [B,H,n_k,d_k],
    V [B,H,n_k,d_v], masses [B,H,n_q] and [B,H,n_k] (nonnegative, summing to one; zero = padding)."""
    b_log = torch.log(beta)[None, :, None, :]
    C1 = torch.einsum("bhnc,hrc->bhnr", Q, Z)
    C2 = torch.einsum("bhnc,hrc->bhnr", K, Z)

    def solve(C, a_log):
        g = torch.zeros_like(b_log)
        f = g_before = None
        for _ in range(T):
            f = eps * (a_log - torch.logsumexp((C + g) / eps, dim=-1, keepdim=True))
            g_before = g
            g = eps * (b_log - torch.logsumexp((C + f) / eps, dim=-2, keepdim=True))
        return f, g, g_before

    with torch.no_grad():
        a1_log = torch.log(mass_q)[..., None]          # -inf for padding
        a2_log = torch.log(mass_k)[..., None]
    _, g1, g1_before = solve(C1, a1_log)
    f2, g2, _ = solve(C2, a2_log)
    gamma2 = torch.exp((C2 + f2 + g2) / eps)                                           # [B,H,n_k,r]
    Yp = torch.einsum("bhnr,bhnc->bhrc", gamma2, V) / beta[None, :, :, None]
    # row i of Diag(mu)^-1 Gamma1: exp((C1 + f1 + g1)/eps) / mu_i with f1 = eps (log mu_i - LSE): mu_i cancels
    rows1 = torch.exp((C1 + g1) / eps - torch.logsumexp((C1 + g1_before) / eps, dim=-1, keepdim=True))
    return torch.einsum("bhnr,bhrc->bhnc", rows1, Yp)


def cross_attention_bwd(Q, K, V, Z, beta, mass_q, mass_k, eps, T, dO):
    """Gradients of <O, dO> with respect to Q, K, V, Z, beta for cross attention with token masses."""
    t = [torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True) for x in (Q, K, V, Z, beta)]
    mq = torch.tensor(np.asarray(mass_q, dtype=np.float64))
    mk = torch.tensor(np.asarray(mass_k, dtype=np.float64))
    O = forward_cross(*t, mq, mk, float(eps), int(T))
    loss = (O * torch.tensor(np.asarray(dO, dtype=np.float64))).sum()
    grads = torch.autograd.grad(loss, t)
    return tuple(g.detach().numpy() for g in grads), O.detach().numpy()
