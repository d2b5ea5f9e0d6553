"""torch.autograd glue for libLOT: differentiable entry points that only marshal arguments.

forward = lot_attention_fwd (or the [CLS] variant), backward = lot_attention_bwd (or its [CLS]
variant); nothing is computed here.  The backward recomputes the forward intermediates inside the
library, so only the inputs are kept between the two calls.

    O = lot_attention(Q, K, V, Z, beta, eps, iters)            # Q, K, V [B,H,n,d], Z [H,r,d], beta [H,r]
    O = lot_attention_cls(Q, K, V, Z, beta, eps, iters, beta_cls)

eps, iters and beta_cls are plain numbers and receive no gradient (the per-problem derivative with
respect to beta_cls is available from lot.lot_attention_cls_bwd).
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


def lot_attention(Q, K, V, Z, beta, eps, iters, path=lot.PATH_AUTO):
    """Differentiable LOT attention: gradients flow to Q, K, V (their dtype) and to Z, beta (float32)."""
    return _LOTAttention.apply(Q, K, V, Z, beta, eps, iters, path)


def lot_attention_cls(Q, K, V, Z, beta, eps, iters, beta_cls, path=lot.PATH_AUTO):
    """Differentiable [CLS] variant (token 0 = [CLS], a softmax row with temperature beta_cls)."""
    return _LOTAttentionCls.apply(Q, K, V, Z, beta, eps, iters, beta_cls, path)
