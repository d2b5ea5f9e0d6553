"""Thin Python binding of libLOT's C ABI (argument marshalling only; see include/lot.h).

Tensors are torch CUDA (ROCm) tensors used as device buffers; every step of the method runs in
the library's own HIP kernels.  There is no fallback: if libLOT.so is missing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libLOT.so")

LOT_F32, LOT_BF16 = 0, 1
PATH_AUTO, PATH_REFERENCE, PATH_FUSED = 0, 1, 2

EXPORTS = ("lot_workspace_bytes", "lot_attention_fwd", "lot_couplings", "lot_attention_fwd_path",
           "lot_couplings_path", "lot_attention_cls_fwd", "lot_attention_cls_fwd_path", "lot_cross_workspace_bytes", "lot_cross_attention_fwd", "lot_cross_attention_fwd_path", "lot_attention_bwd_workspace_bytes", "lot_attention_bwd", "lot_attention_bwd_path",
           "lot_attention_cls_bwd", "lot_attention_cls_bwd_path",
           "lot_cross_attention_bwd_workspace_bytes", "lot_cross_attention_bwd", "lot_cross_attention_bwd_path",
           "lot_workspace_status", "lot_strerror", "lot_version")


class lot_shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("n", ctypes.c_int32),
                ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("r", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32)]


class lot_xshape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("n_q", ctypes.c_int32), ("n_k", ctypes.c_int32),
                ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("r", ctypes.c_int32),
                ("io_dtype", ctypes.c_int32)]


class LotError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libLOT error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libLOT.so is not built (run `python -m paper_2509_23436_amd.build`); "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, fp, sz = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t
        sp = ctypes.POINTER(lot_shape)
        L.lot_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(sz)]
        L.lot_attention_fwd.argtypes = [sp, vp, vp, vp, fp, fp, ctypes.c_float, ctypes.c_int, vp, vp, sz, vp]
        L.lot_attention_fwd_path.argtypes = L.lot_attention_fwd.argtypes + [ctypes.c_int]
        L.lot_couplings.argtypes = [sp, vp, vp, fp, fp, ctypes.c_float, ctypes.c_int, fp, fp, vp, sz, vp]
        L.lot_couplings_path.argtypes = L.lot_couplings.argtypes + [ctypes.c_int]
        L.lot_workspace_status.argtypes = [vp]
        L.lot_strerror.argtypes = [ctypes.c_int]
        L.lot_strerror.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name != "lot_strerror":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code):
    if code != 0:
        raise LotError(code, lib().lot_strerror(code).decode())


def _shape_of(Q, V, Z) -> lot_shape:
    B, H, n, d_k = Q.shape
    if Q.dtype == torch.float32:
        dt = LOT_F32
    elif Q.dtype == torch.bfloat16:
        dt = LOT_BF16
    else:
        raise TypeError("Q, K, V must be float32 or bfloat16")
    d_v = V.shape[3] if V is not None else d_k
    return lot_shape(B, H, n, d_k, d_v, Z.shape[1], dt)


def lot_workspace_bytes(shape: lot_shape, iters: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lot_workspace_bytes(ctypes.byref(shape), int(iters), ctypes.byref(out)))
    return out.value


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _require(t, name, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(name + " must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(name + " must be " + str(dtype))


def alloc_workspace(shape: lot_shape, iters: int, device="cuda") -> torch.Tensor:
    return torch.empty(lot_workspace_bytes(shape, iters), dtype=torch.uint8, device=device)


def lot_attention_fwd(Q, K, V, Z, beta, eps, iters, out=None, workspace=None, path=PATH_AUTO):
    """out[B,H,n,d_v] = LOTAttn(Q, K, V) with pivot measure (Z[H,r,d_k], beta[H,r])."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    shape = _shape_of(Q, V, Z)
    if out is None:
        out = torch.empty_like(V)
    _require(out, "out", Q.dtype)
    if workspace is None:
        workspace = alloc_workspace(shape, iters, Q.device)
    _check(lib().lot_attention_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                        ctypes.c_float(eps), int(iters), _ptr(out), _ptr(workspace),
                                        workspace.numel(), _stream(), int(path)))
    return out


def lot_couplings(Q, K, Z, beta, eps, iters, workspace=None, path=PATH_AUTO):
    """(gamma1[B,H,n,r], gamma2[B,H,r,n]) in float32."""
    for t, nm in ((Q, "Q"), (K, "K")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    shape = _shape_of(Q, None, Z)
    B, H, n, _ = Q.shape
    r = Z.shape[1]
    g1 = torch.empty((B, H, n, r), dtype=torch.float32, device=Q.device)
    g2 = torch.empty((B, H, r, n), dtype=torch.float32, device=Q.device)
    if workspace is None:
        workspace = alloc_workspace(shape, iters, Q.device)
    _check(lib().lot_couplings_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(Z), _ptr(beta),
                                    ctypes.c_float(eps), int(iters), _ptr(g1), _ptr(g2), _ptr(workspace),
                                    workspace.numel(), _stream(), int(path)))
    return g1, g2


def lot_workspace_status(workspace) -> int:
    return lib().lot_workspace_status(_ptr(workspace))


def lot_version() -> int:
    return lib().lot_version()


def lot_attention_bwd_workspace_bytes(shape: lot_shape, iters: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().lot_attention_bwd_workspace_bytes(ctypes.byref(shape), int(iters), ctypes.byref(out)))
    return out.value


def lot_attention_bwd(Q, K, V, Z, beta, eps, iters, dO, workspace=None, path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta) of <LOTAttn(Q, K, V), dO>; dZ and dbeta are summed over the batch."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    if dO.shape != V.shape:
        raise ValueError("dO must have the shape of V")
    shape = _shape_of(Q, V, Z)
    need = lot_attention_bwd_workspace_bytes(shape, iters)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    _require(workspace, "workspace", torch.uint8)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    _check(lib().lot_attention_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                        ctypes.c_float(eps), int(iters), _ptr(dO),
                                        _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta),
                                        _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta


def lot_attention_cls_fwd(Q, K, V, Z, beta, eps, iters, beta_cls, out=None, workspace=None, path=PATH_AUTO):
    """LOT attention among tokens 1..n-1 plus a softmax row (temperature beta_cls) for token 0 ([CLS])."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    shape = _shape_of(Q, V, Z)
    if out is None:
        out = torch.empty_like(V)
    _require(out, "out", Q.dtype)
    if workspace is None:
        workspace = alloc_workspace(shape, iters, Q.device)
    _require(workspace, "workspace", torch.uint8)
    _check(lib().lot_attention_cls_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                            ctypes.c_float(eps), int(iters), ctypes.c_float(beta_cls), _ptr(out),
                                            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return out


def lot_attention_cls_bwd(Q, K, V, Z, beta, eps, iters, beta_cls, dO, workspace=None, path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta, dbeta_cls[B,H]) of <lot_attention_cls_fwd(...), dO>."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    if dO.shape != V.shape:
        raise ValueError("dO must have the shape of V")
    shape = _shape_of(Q, V, Z)
    if workspace is None:
        workspace = torch.empty(lot_attention_bwd_workspace_bytes(shape, iters), dtype=torch.uint8, device=Q.device)
    _require(workspace, "workspace", torch.uint8)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    dbeta_cls = torch.empty(Q.shape[:2], dtype=torch.float32, device=Q.device)
    _check(lib().lot_attention_cls_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                            ctypes.c_float(eps), int(iters), ctypes.c_float(beta_cls), _ptr(dO),
                                            _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta), _ptr(dbeta_cls),
                                            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta, dbeta_cls


def lot_cross_attention_fwd(Q, K, V, Z, beta, eps, iters, mass_q=None, mass_k=None, out=None, workspace=None,
                            path=PATH_AUTO):
    """Cross attention with optional token masses: Q [B,H,n_q,d], K [B,H,n_k,d], V [B,H,n_k,d_v]."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    B, H, n_q, d_k = Q.shape
    n_k, d_v = K.shape[2], V.shape[3]
    dt = LOT_F32 if Q.dtype == torch.float32 else LOT_BF16
    shape = lot_xshape(B, H, n_q, n_k, d_k, d_v, Z.shape[1], dt)
    for m, nm, n in ((mass_q, "mass_q", n_q), (mass_k, "mass_k", n_k)):
        if m is not None:
            _require(m, nm, torch.float32)
            if tuple(m.shape) != (B, H, n):
                raise ValueError(nm + " must be [B, H, n]")
    if out is None:
        out = torch.empty((B, H, n_q, d_v), dtype=Q.dtype, device=Q.device)
    need = ctypes.c_size_t(0)
    _check(lib().lot_cross_workspace_bytes(ctypes.byref(shape), int(iters), ctypes.byref(need)))
    if workspace is None:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=Q.device)
    _require(workspace, "workspace", torch.uint8)
    null = ctypes.c_void_p(0)
    _check(lib().lot_cross_attention_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                              _ptr(mass_q) if mass_q is not None else null,
                                              _ptr(mass_k) if mass_k is not None else null,
                                              ctypes.c_float(eps), int(iters), _ptr(out),
                                              _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(),
                                              int(path)))
    return out


def lot_cross_attention_bwd(Q, K, V, Z, beta, eps, iters, dO, mass_q=None, mass_k=None, workspace=None,
                            path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta) of <lot_cross_attention_fwd(...), dO>; the masses are not differentiated."""
    for t, nm in ((Q, "Q"), (K, "K"), (V, "V"), (dO, "dO")):
        _require(t, nm, Q.dtype)
    _require(Z, "Z", torch.float32)
    _require(beta, "beta", torch.float32)
    B, H, n_q, d_k = Q.shape
    n_k, d_v = K.shape[2], V.shape[3]
    if tuple(dO.shape) != (B, H, n_q, d_v):
        raise ValueError("dO must be [B, H, n_q, d_v]")
    dt = LOT_F32 if Q.dtype == torch.float32 else LOT_BF16
    shape = lot_xshape(B, H, n_q, n_k, d_k, d_v, Z.shape[1], dt)
    for m, nm, n in ((mass_q, "mass_q", n_q), (mass_k, "mass_k", n_k)):
        if m is not None:
            _require(m, nm, torch.float32)
            if tuple(m.shape) != (B, H, n):
                raise ValueError(nm + " must be [B, H, n]")
    need = ctypes.c_size_t(0)
    _check(lib().lot_cross_attention_bwd_workspace_bytes(ctypes.byref(shape), int(iters), ctypes.byref(need)))
    if workspace is None:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=Q.device)
    _require(workspace, "workspace", torch.uint8)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    null = ctypes.c_void_p(0)
    _check(lib().lot_cross_attention_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                         _ptr(mass_q) if mass_q is not None else null,
                                         _ptr(mass_k) if mass_k is not None else null,
                                         ctypes.c_float(eps), int(iters), _ptr(dO),
                                         _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta),
                                         _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta
