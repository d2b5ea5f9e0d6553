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

Workspaces: one per (device, call kind, shape, iters, path), allocated at the first call and reused, so a
training step allocates nothing for them after its first iteration.  Calls that share a workspace must be
on one stream (torch's current stream at each call); use the functions of `lot` with workspaces of your
own to run the same shape on several streams at once.

Failed waits: after every call the two status words of its workspace are copied to pinned host memory
on the same stream (no synchronisation); every later call first looks at the copies that have arrived
and raises if one of them reports a wait between workgroups that gave up (see include/lot.h; the rows
such a call left unwritten are NaN in any case).  `check_pending(wait=True)` waits for all of them.
After such a report the calls that were left to choose their kernels (path = lot.PATH_AUTO) run on
lot.PATH_STEPWISE where the shape allows it: the same tile kernels, one launch per Sinkhorn pass, no waits
between workgroups, so whatever shares the device cannot make them fail again (`stepwise_after_failure`).
"""
import torch

from . import lot

_workspaces = {}
_pending = []
stepwise_after_failure = False      # set by check_pending at the first reported failure; may be reset by the caller


def _workspace(kind, size_fn, shape_key, device, shape, iters, path):
    key = (str(device), kind, shape_key, int(iters), int(path))
    ws = _workspaces.get(key)
    if ws is None:
        ws = torch.empty(size_fn(shape, iters, path), dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def check_pending(wait=False):
    """Raises RuntimeError if a finished call reported a wait that gave up; with wait=True, waits for
    every outstanding status copy first (each waits for its own point of its stream only)."""
    still = []
    bad = None
    for what, probe in _pending:
        if wait or probe.ready():
            if probe.failed() and bad is None:
                bad = what
        else:
            still.append((what, probe))
    _pending[:] = still
    if bad is not None:
        global stepwise_after_failure
        stepwise_after_failure = True
        raise RuntimeError("libLOT: a wait between workgroups gave up during %s (another stream's kernel held "
                           "compute units while it started?); its result is marked with NaN" % bad)


def _resolve(path, shape, iters, fwd_size, bwd_size):
    """AUTO -> STEPWISE once a wait has failed in this process, where both passes support the shape on it."""
    if path != lot.PATH_AUTO or not stepwise_after_failure:
        return path
    try:
        fwd_size(shape, iters, lot.PATH_STEPWISE)
        bwd_size(shape, iters, lot.PATH_STEPWISE)
    except RuntimeError:
        return path
    return lot.PATH_STEPWISE


def _after(what, ws):
    _pending.append((what, lot.StatusProbe(ws)))


def _fwd_shape(Q, V, Z):
    return lot._shape_of(Q, V, Z), (tuple(Q.shape), V.shape[3], Z.shape[1], str(Q.dtype))


def _cross_shape(Q, K, V, Z):
    B, H, n_q, d_k = Q.shape
    shape = lot.lot_xshape(B, H, n_q, K.shape[2], d_k, V.shape[3], Z.shape[1], lot._dtype_code(Q))
    return shape, (tuple(Q.shape), K.shape[2], V.shape[3], Z.shape[1], str(Q.dtype))


class _LOTAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        ctx.save_for_backward(Q, K, V, Z, beta)
        check_pending()
        lot._dims(Q, K, V, Z, beta)
        shape, key = _fwd_shape(Q, V, Z)
        path = _resolve(path, shape, iters, lot.lot_workspace_bytes, lot.lot_attention_bwd_workspace_bytes)
        ctx.cfg = (float(eps), int(iters), int(path))
        ws = _workspace("fwd", lot.lot_workspace_bytes, key, Q.device, shape, iters, path)
        out = lot.lot_attention_fwd(Q, K, V, Z, beta, eps, iters, workspace=ws, path=path)
        _after("lot_attention (forward)", ws)
        return out

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        eps, iters, path = ctx.cfg
        check_pending()
        shape, key = _fwd_shape(Q, V, Z)
        ws = _workspace("bwd", lot.lot_attention_bwd_workspace_bytes, key, Q.device, shape, iters, path)
        grads = lot.lot_attention_bwd(Q, K, V, Z, beta, eps, iters, dO.contiguous().to(Q.dtype), workspace=ws, path=path)
        _after("lot_attention (backward)", ws)
        return (*grads, None, None, None)


class _LOTAttentionCls(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, beta_cls, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        ctx.save_for_backward(Q, K, V, Z, beta)
        check_pending()
        lot._dims(Q, K, V, Z, beta)
        shape, key = _fwd_shape(Q, V, Z)
        path = _resolve(path, shape, iters, lot.lot_workspace_bytes, lot.lot_attention_bwd_workspace_bytes)
        ctx.cfg = (float(eps), int(iters), float(beta_cls), int(path))
        ws = _workspace("fwd", lot.lot_workspace_bytes, key, Q.device, shape, iters, path)
        out = lot.lot_attention_cls_fwd(Q, K, V, Z, beta, eps, iters, beta_cls, workspace=ws, path=path)
        _after("lot_attention_cls (forward)", ws)
        return out

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        eps, iters, beta_cls, path = ctx.cfg
        check_pending()
        shape, key = _fwd_shape(Q, V, Z)
        ws = _workspace("bwd", lot.lot_attention_bwd_workspace_bytes, key, Q.device, shape, iters, path)
        grads = lot.lot_attention_cls_bwd(Q, K, V, Z, beta, eps, iters, beta_cls, dO.contiguous().to(Q.dtype),
                                          workspace=ws, path=path)
        _after("lot_attention_cls (backward)", ws)
        return (*grads[:5], None, None, None, None)


class _LOTCrossAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, Z, beta, eps, iters, mass_q, mass_k, path):
        Q, K, V, Z, beta = (t.contiguous() for t in (Q, K, V, Z, beta))
        mass_q = None if mass_q is None else mass_q.contiguous()
        mass_k = None if mass_k is None else mass_k.contiguous()
        ctx.save_for_backward(Q, K, V, Z, beta)
        ctx.masses = (mass_q, mass_k)
        check_pending()
        lot._dims(Q, K, V, Z, beta, cross=True)
        shape, key = _cross_shape(Q, K, V, Z)
        path = _resolve(path, shape, iters, lot.lot_cross_workspace_bytes, lot.lot_cross_attention_bwd_workspace_bytes)
        ctx.cfg = (float(eps), int(iters), int(path))
        ws = _workspace("xfwd", lot.lot_cross_workspace_bytes, key, Q.device, shape, iters, path)
        out = lot.lot_cross_attention_fwd(Q, K, V, Z, beta, eps, iters, mass_q=mass_q, mass_k=mass_k, workspace=ws,
                                          path=path)
        _after("lot_cross_attention (forward)", ws)
        return out

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, Z, beta = ctx.saved_tensors
        mass_q, mass_k = ctx.masses
        eps, iters, path = ctx.cfg
        check_pending()
        shape, key = _cross_shape(Q, K, V, Z)
        ws = _workspace("xbwd", lot.lot_cross_attention_bwd_workspace_bytes, key, Q.device, shape, iters, path)
        grads = lot.lot_cross_attention_bwd(Q, K, V, Z, beta, eps, iters, dO.contiguous().to(Q.dtype),
                                            mass_q=mass_q, mass_k=mass_k, workspace=ws, path=path)
        _after("lot_cross_attention (backward)", ws)
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
