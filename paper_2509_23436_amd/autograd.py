"""torch.autograd glue for libLOT: differentiable entry points that only marshal arguments.

forward = lot_attention_fwd (or the [CLS] variant), backward = lot_attention_bwd (or its [CLS]
variant); nothing is computed here.  The backward recomputes the forward intermediates inside the
library, so only the inputs are kept between the two calls.

    O = lot_attention(Q, K, V, Z, beta, eps, iters)            # Q, K, V [B,H,n,d], Z [H,r,d], beta [H,r]
    O = lot_attention_cls(Q, K, V, Z, beta, eps, iters, beta_cls)
    O = lot_cross_attention(Q, K, V, Z, beta, eps, iters, mass_q=None, mass_k=None)   # Q [B,H,n_q,d], K, V [B,H,n_k,.]

eps, iters and beta_cls are plain numbers and receive no gradient (the per-problem derivative with
respect to beta_cls is available from lot.lot_attention_cls_bwd); the token masses of cross attention
are data (a padding mask), not differentiated.
"""
import torch

from . import lot


class _LOTAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        ctx.save_for_backward(Q, K, V, Z, beta)
        ctx.cfg = (float(eps), int(iters), int(path))
        return lot.lot_attention_fwd(Q, K, V, Z, beta, eps, iters, path=path)

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        eps, iters, path = ctx.cfg
        grads = lot.lot_attention_bwd(Q, K, V, Z, beta, eps, iters, dO.contiguous().to(Q.dtype), path=path)
        return (*grads, None, None, None)


class _LOTAttentionCls(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, beta_cls, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        ctx.save_for_backward(Q, K, V, Z, beta)
        ctx.cfg = (float(eps), int(iters), float(beta_cls), int(path))
        return lot.lot_attention_cls_fwd(Q, K, V, Z, beta, eps, iters, beta_cls, path=path)

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        eps, iters, beta_cls, path = ctx.cfg
        grads = lot.lot_attention_cls_bwd(Q, K, V, Z, beta, eps, iters, beta_cls, dO.contiguous().to(Q.dtype), path=path)
        return (*grads[:5], None, None, None, None)


class _LOTCrossAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, mass_q, mass_k, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        mass_q = None if mass_q is None else mass_q.contiguous()
        mass_k = None if mass_k is None else mass_k.contiguous()
        ctx.save_for_backward(Q, K, V, Z, beta)
        ctx.masses = (mass_q, mass_k)
        ctx.cfg = (float(eps), int(iters), int(path))
        return lot.lot_cross_attention_fwd(Q, K, V, Z, beta, eps, iters, mass_q=mass_q, mass_k=mass_k, path=path)

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        mass_q, mass_k = ctx.masses
        eps, iters, path = ctx.cfg
        grads = lot.lot_cross_attention_bwd(Q, K, V, Z, beta, eps, iters, dO.contiguous().to(Q.dtype),
                                            mass_q=mass_q, mass_k=mass_k, path=path)
        return (*grads, None, None, None, None, None)


def lot_attention(Q, K, V, Z, beta, eps, iters, path=lot.PATH_AUTO):
    """Differentiable LOT attention: gradients flow to Q, K, V (their dtype) and to Z, beta (float32)."""
    return _LOTAttention.apply(Q, K, V, Z, beta, eps, iters, path)


def lot_attention_cls(Q, K, V, Z, beta, eps, iters, beta_cls, path=lot.PATH_AUTO):
    """Differentiable [CLS] variant (token 0 = [CLS], a softmax row with temperature beta_cls)."""
    return _LOTAttentionCls.apply(Q, K, V, Z, beta, eps, iters, beta_cls, path)


def lot_cross_attention(Q, K, V, Z, beta, eps, iters, mass_q=None, mass_k=None, path=lot.PATH_AUTO):
    """Differentiable cross attention with optional token masses [B,H,n_q], [B,H,n_k] (zero = padding)."""
    return _LOTCrossAttention.apply(Q, K, V, Z, beta, eps, iters, mass_q, mass_k, path)
