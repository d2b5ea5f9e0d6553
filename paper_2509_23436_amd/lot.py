"""Thin Python binding of libLOT's C ABI (argument marshalling only; see include/lot.h).

Tensors are torch CUDA (ROCm) tensors used as device buffers; every step of the method runs in
the library's own HIP kernels.  There is no fallback: if libLOT.so is missing this module raises.

The C ABI sees only pointers, so every shape, dtype and device is checked here, on the host, before a
call: a tensor shorter than the shape says would make a kernel read or write past its allocation.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libLOT.so")

LOT_F32, LOT_BF16 = 0, 1
PATH_AUTO, PATH_REFERENCE, PATH_FUSED, PATH_STEPWISE = 0, 1, 2, 3
KNOB_SPIN_LIMIT, KNOB_RESHIFT_BITS, KNOB_BWD_ASSEMBLE_BY_ITERATION, KNOB_BWD_SWEEP_LAUNCHES = 0, 1, 2, 3
KNOB_FWD_STREAMING, KNOB_FWD_DRIFT_LIMIT, KNOB_GROUPED_ONE_LAUNCH_TILES, KNOB_BWD_SWEEP_RECOMPUTE = 4, 5, 6, 7
ERR_SYNC = -10

EXPORTS = ("lot_workspace_bytes", "lot_workspace_bytes_path", "lot_couplings_workspace_bytes",
           "lot_attention_fwd", "lot_attention_fwd_path", "lot_attention_fwd_static", "lot_static_scratch_bytes",
           "lot_forward_kernels",
           "lot_couplings", "lot_couplings_path",
           "lot_attention_cls_fwd", "lot_attention_cls_fwd_path",
           "lot_cross_workspace_bytes", "lot_cross_workspace_bytes_path",
           "lot_cross_attention_fwd", "lot_cross_attention_fwd_path",
           "lot_attention_bwd_workspace_bytes", "lot_attention_bwd_workspace_bytes_path",
           "lot_attention_bwd", "lot_attention_bwd_path",
           "lot_attention_cls_bwd", "lot_attention_cls_bwd_path",
           "lot_cross_attention_bwd_workspace_bytes", "lot_cross_attention_bwd_workspace_bytes_path",
           "lot_cross_attention_bwd", "lot_cross_attention_bwd_path",
           "lot_workspace_status", "lot_workspace_status_async", "lot_status_words", "lot_debug_set",
           "lot_strerror", "lot_version")


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
        vp, sz, ci, cf = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
        sp, xp, szp = ctypes.POINTER(lot_shape), ctypes.POINTER(lot_xshape), ctypes.POINTER(ctypes.c_size_t)
        L.lot_workspace_bytes.argtypes = [sp, ci, szp]
        L.lot_workspace_bytes_path.argtypes = [sp, ci, ci, szp]
        L.lot_couplings_workspace_bytes.argtypes = [sp, ci, ci, szp]
        L.lot_attention_bwd_workspace_bytes.argtypes = [sp, ci, szp]
        L.lot_attention_bwd_workspace_bytes_path.argtypes = [sp, ci, ci, szp]
        L.lot_cross_workspace_bytes.argtypes = [xp, ci, szp]
        L.lot_cross_workspace_bytes_path.argtypes = [xp, ci, ci, szp]
        L.lot_cross_attention_bwd_workspace_bytes.argtypes = [xp, ci, szp]
        L.lot_cross_attention_bwd_workspace_bytes_path.argtypes = [xp, ci, ci, szp]
        L.lot_attention_fwd.argtypes = [sp, vp, vp, vp, vp, vp, cf, ci, vp, vp, sz, vp]
        L.lot_attention_fwd_path.argtypes = L.lot_attention_fwd.argtypes + [ci]
        L.lot_forward_kernels.argtypes = [sp, ci, ci, ctypes.POINTER(ctypes.c_int)]
        L.lot_attention_fwd_static.argtypes = [sp, vp, vp, vp, vp, vp, cf, ci, vp, vp]
        L.lot_static_scratch_bytes.argtypes = []
        L.lot_static_scratch_bytes.restype = sz
        L.lot_couplings.argtypes = [sp, vp, vp, vp, vp, cf, ci, vp, vp, vp, sz, vp]
        L.lot_couplings_path.argtypes = L.lot_couplings.argtypes + [ci]
        L.lot_attention_cls_fwd.argtypes = [sp, vp, vp, vp, vp, vp, cf, ci, cf, vp, vp, sz, vp]
        L.lot_attention_cls_fwd_path.argtypes = L.lot_attention_cls_fwd.argtypes + [ci]
        L.lot_cross_attention_fwd.argtypes = [xp, vp, vp, vp, vp, vp, vp, vp, cf, ci, vp, vp, sz, vp]
        L.lot_cross_attention_fwd_path.argtypes = L.lot_cross_attention_fwd.argtypes + [ci]
        L.lot_attention_bwd.argtypes = [sp, vp, vp, vp, vp, vp, cf, ci, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lot_attention_bwd_path.argtypes = L.lot_attention_bwd.argtypes + [ci]
        L.lot_attention_cls_bwd.argtypes = [sp, vp, vp, vp, vp, vp, cf, ci, cf, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lot_attention_cls_bwd_path.argtypes = L.lot_attention_cls_bwd.argtypes + [ci]
        L.lot_cross_attention_bwd.argtypes = [xp, vp, vp, vp, vp, vp, vp, vp, cf, ci, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lot_cross_attention_bwd_path.argtypes = L.lot_cross_attention_bwd.argtypes + [ci]
        L.lot_workspace_status.argtypes = [vp]
        L.lot_workspace_status_async.argtypes = [vp, vp, vp]
        L.lot_status_words.argtypes = [vp]
        L.lot_debug_set.argtypes = [ci, ctypes.c_longlong]
        L.lot_strerror.argtypes = [ci]
        L.lot_strerror.restype = ctypes.c_char_p
        L.lot_version.argtypes = []
        for name in EXPORTS:
            if name not in ("lot_strerror", "lot_static_scratch_bytes"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(code):
    if code != 0:
        raise LotError(code, lib().lot_strerror(code).decode())


# ---------------------------------------------------------------------------------------------
# host-side checks: the C ABI sees only pointers
# ---------------------------------------------------------------------------------------------
def _dtype_code(t):
    if t.dtype == torch.float32:
        return LOT_F32
    if t.dtype == torch.bfloat16:
        return LOT_BF16
    raise TypeError("Q, K, V must be float32 or bfloat16")


def _require(t, name, dtype, shape, device):
    """`t` is a contiguous tensor of exactly this dtype and shape on this device (a CUDA/ROCm device)."""
    if not isinstance(t, torch.Tensor):
        raise TypeError(name + " must be a torch tensor")
    if t.dtype != dtype:
        raise TypeError("%s must be %s, not %s" % (name, dtype, t.dtype))
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, not %s" % (name, tuple(shape), tuple(t.shape)))
    if t.device != device:
        raise ValueError("%s must be on %s, not %s" % (name, device, t.device))
    if not t.is_contiguous():
        raise ValueError(name + " must be contiguous")


def _on_current_device(device):
    """The kernels are launched on torch's current stream, which belongs to the current device."""
    if device.type != "cuda":
        raise ValueError("the tensors must be on a GPU device (there is no CPU path), not on %s" % device)
    if device.index is not None and device.index != torch.cuda.current_device():
        raise ValueError("the tensors are on %s but the current device is %d" % (device, torch.cuda.current_device()))


def _dims(Q, K, V, Z, beta, cross=False):
    """Checks the five inputs against each other and returns (B, H, n_q, n_k, d_k, d_v, r, dtype code)."""
    if not isinstance(Q, torch.Tensor) or Q.dim() != 4:
        raise ValueError("Q must be a [B, H, n, d_k] tensor")
    code = _dtype_code(Q)
    B, H, n_q, d_k = Q.shape
    if not isinstance(K, torch.Tensor) or K.dim() != 4:
        raise ValueError("K must be a [B, H, n, d_k] tensor")
    n_k = K.shape[2] if cross else n_q
    _require(Q, "Q", Q.dtype, (B, H, n_q, d_k), Q.device)
    _require(K, "K", Q.dtype, (B, H, n_k, d_k), Q.device)
    d_v = d_k
    if V is not None:
        if not isinstance(V, torch.Tensor) or V.dim() != 4:
            raise ValueError("V must be a [B, H, n, d_v] tensor")
        d_v = V.shape[3]
        _require(V, "V", Q.dtype, (B, H, n_k, d_v), Q.device)
    if not isinstance(Z, torch.Tensor) or Z.dim() != 3:
        raise ValueError("Z must be a [H, r, d_k] tensor")
    r = Z.shape[1]
    _require(Z, "Z", torch.float32, (H, r, d_k), Q.device)
    _require(beta, "beta", torch.float32, (H, r), Q.device)
    return B, H, n_q, n_k, d_k, d_v, r, code


def _shape_of(Q, V, Z) -> lot_shape:
    B, H, n, d_k = Q.shape
    d_v = V.shape[3] if V is not None else d_k
    return lot_shape(B, H, n, d_k, d_v, Z.shape[1], _dtype_code(Q))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else 0)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _workspace(workspace, need, device):
    """The last host-side step before a call: the device is checked here, after every shape and dtype."""
    _on_current_device(device)
    if workspace is None:
        return torch.empty(need, dtype=torch.uint8, device=device)
    if not isinstance(workspace, torch.Tensor) or workspace.dtype != torch.uint8 or workspace.dim() != 1:
        raise TypeError("workspace must be a one-dimensional uint8 tensor")
    if workspace.device != device or not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous and on the inputs' device")
    if workspace.numel() < need:
        raise ValueError("workspace holds %d bytes, this call needs %d" % (workspace.numel(), need))
    return workspace


def _sized(fn, shape, iters, *path):
    out = ctypes.c_size_t(0)
    _check(fn(ctypes.byref(shape), int(iters), *[int(p) for p in path], ctypes.byref(out)))
    return out.value


# ---------------------------------------------------------------------------------------------
# workspace sizes
# ---------------------------------------------------------------------------------------------
def lot_workspace_bytes(shape: lot_shape, iters: int, path=PATH_AUTO) -> int:
    return _sized(lib().lot_workspace_bytes_path, shape, iters, path)


def lot_couplings_workspace_bytes(shape: lot_shape, iters: int, path=PATH_AUTO) -> int:
    return _sized(lib().lot_couplings_workspace_bytes, shape, iters, path)


def lot_attention_bwd_workspace_bytes(shape: lot_shape, iters: int, path=PATH_AUTO) -> int:
    return _sized(lib().lot_attention_bwd_workspace_bytes_path, shape, iters, path)


def lot_cross_workspace_bytes(shape: lot_xshape, iters: int, path=PATH_AUTO) -> int:
    return _sized(lib().lot_cross_workspace_bytes_path, shape, iters, path)


def lot_cross_attention_bwd_workspace_bytes(shape: lot_xshape, iters: int, path=PATH_AUTO) -> int:
    return _sized(lib().lot_cross_attention_bwd_workspace_bytes_path, shape, iters, path)


def alloc_workspace(shape: lot_shape, iters: int, device="cuda", path=PATH_AUTO, couplings=False) -> torch.Tensor:
    """A workspace for lot_attention_fwd (and, with couplings=True, large enough for lot_couplings too)."""
    need = lot_workspace_bytes(shape, iters, path)
    if couplings:
        need = max(need, lot_couplings_workspace_bytes(shape, iters, path))
    return torch.empty(need, dtype=torch.uint8, device=device)


# ---------------------------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------------------------
def lot_attention_fwd(Q, K, V, Z, beta, eps, iters, out=None, workspace=None, path=PATH_AUTO):
    """out[B,H,n,d_v] = LOTAttn(Q, K, V) with pivot measure (Z[H,r,d_k], beta[H,r])."""
    B, H, n, _, d_k, d_v, r, code = _dims(Q, K, V, Z, beta)
    shape = lot_shape(B, H, n, d_k, d_v, r, code)
    if out is None:
        out = torch.empty_like(V)
    _require(out, "out", Q.dtype, (B, H, n, d_v), Q.device)
    workspace = _workspace(workspace, lot_workspace_bytes(shape, iters, path), Q.device)
    _check(lib().lot_attention_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                        ctypes.c_float(eps), int(iters), _ptr(out), _ptr(workspace),
                                        workspace.numel(), _stream(), int(path)))
    return out


KERNELS = ("plain", "streaming", "kept_workgroup", "kept_wavefront", "grouped")


def lot_forward_kernels(shape: lot_shape, iters: int, path=PATH_AUTO) -> str:
    """The family of kernels lot_attention_fwd would run for this shape on the current device."""
    out = ctypes.c_int(-1)
    _check(lib().lot_forward_kernels(ctypes.byref(shape), int(iters), int(path), ctypes.byref(out)))
    return KERNELS[out.value]


def lot_static_scratch_bytes() -> int:
    return int(lib().lot_static_scratch_bytes())


def lot_attention_fwd_static(Q, K, V, Z, beta, eps, iters, out):
    """lot_attention_fwd for callers that cannot allocate: no workspace argument (the library's own
    fixed scratch array is used), `out` is required."""
    B, H, n, _, d_k, d_v, r, code = _dims(Q, K, V, Z, beta)
    shape = lot_shape(B, H, n, d_k, d_v, r, code)
    _require(out, "out", Q.dtype, (B, H, n, d_v), Q.device)
    _on_current_device(Q.device)
    _check(lib().lot_attention_fwd_static(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                          ctypes.c_float(eps), int(iters), _ptr(out), _stream()))
    return out


def lot_couplings(Q, K, Z, beta, eps, iters, workspace=None, path=PATH_AUTO):
    """(gamma1[B,H,n,r], gamma2[B,H,r,n]) in float32."""
    B, H, n, _, d_k, _, r, code = _dims(Q, K, None, Z, beta)
    shape = lot_shape(B, H, n, d_k, d_k, r, code)
    g1 = torch.empty((B, H, n, r), dtype=torch.float32, device=Q.device)
    g2 = torch.empty((B, H, r, n), dtype=torch.float32, device=Q.device)
    workspace = _workspace(workspace, lot_couplings_workspace_bytes(shape, iters, path), Q.device)
    _check(lib().lot_couplings_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(Z), _ptr(beta),
                                    ctypes.c_float(eps), int(iters), _ptr(g1), _ptr(g2), _ptr(workspace),
                                    workspace.numel(), _stream(), int(path)))
    return g1, g2


def lot_attention_cls_fwd(Q, K, V, Z, beta, eps, iters, beta_cls, out=None, workspace=None, path=PATH_AUTO):
    """LOT attention among tokens 1..n-1 plus a softmax row (temperature beta_cls) for token 0 ([CLS])."""
    B, H, n, _, d_k, d_v, r, code = _dims(Q, K, V, Z, beta)
    shape = lot_shape(B, H, n, d_k, d_v, r, code)
    if out is None:
        out = torch.empty_like(V)
    _require(out, "out", Q.dtype, (B, H, n, d_v), Q.device)
    workspace = _workspace(workspace, lot_workspace_bytes(shape, iters, path), Q.device)
    _check(lib().lot_attention_cls_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                            ctypes.c_float(eps), int(iters), ctypes.c_float(beta_cls), _ptr(out),
                                            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return out


def _masses(mass_q, mass_k, B, H, n_q, n_k, device):
    for m, nm, n in ((mass_q, "mass_q", n_q), (mass_k, "mass_k", n_k)):
        if m is not None:
            _require(m, nm, torch.float32, (B, H, n), device)


def lot_cross_attention_fwd(Q, K, V, Z, beta, eps, iters, mass_q=None, mass_k=None, out=None, workspace=None,
                            path=PATH_AUTO):
    """Cross attention with optional token masses: Q [B,H,n_q,d], K [B,H,n_k,d], V [B,H,n_k,d_v]."""
    B, H, n_q, n_k, d_k, d_v, r, code = _dims(Q, K, V, Z, beta, cross=True)
    shape = lot_xshape(B, H, n_q, n_k, d_k, d_v, r, code)
    _masses(mass_q, mass_k, B, H, n_q, n_k, Q.device)
    if out is None:
        out = torch.empty((B, H, n_q, d_v), dtype=Q.dtype, device=Q.device)
    _require(out, "out", Q.dtype, (B, H, n_q, d_v), Q.device)
    workspace = _workspace(workspace, lot_cross_workspace_bytes(shape, iters, path), Q.device)
    _check(lib().lot_cross_attention_fwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                              _ptr(mass_q), _ptr(mass_k),
                                              ctypes.c_float(eps), int(iters), _ptr(out),
                                              _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(),
                                              int(path)))
    return out


# ---------------------------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------------------------
def lot_attention_bwd(Q, K, V, Z, beta, eps, iters, dO, workspace=None, path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta) of <LOTAttn(Q, K, V), dO>; dZ and dbeta are summed over the batch."""
    B, H, n, _, d_k, d_v, r, code = _dims(Q, K, V, Z, beta)
    _require(dO, "dO", Q.dtype, (B, H, n, d_v), Q.device)
    shape = lot_shape(B, H, n, d_k, d_v, r, code)
    workspace = _workspace(workspace, lot_attention_bwd_workspace_bytes(shape, iters, path), Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    _check(lib().lot_attention_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                        ctypes.c_float(eps), int(iters), _ptr(dO),
                                        _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta),
                                        _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta


def lot_attention_cls_bwd(Q, K, V, Z, beta, eps, iters, beta_cls, dO, workspace=None, path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta, dbeta_cls[B,H]) of <lot_attention_cls_fwd(...), dO>."""
    B, H, n, _, d_k, d_v, r, code = _dims(Q, K, V, Z, beta)
    _require(dO, "dO", Q.dtype, (B, H, n, d_v), Q.device)
    shape = lot_shape(B, H, n, d_k, d_v, r, code)
    workspace = _workspace(workspace, lot_attention_bwd_workspace_bytes(shape, iters, path), Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    dbeta_cls = torch.empty((B, H), dtype=torch.float32, device=Q.device)
    _check(lib().lot_attention_cls_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                            ctypes.c_float(eps), int(iters), ctypes.c_float(beta_cls), _ptr(dO),
                                            _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta), _ptr(dbeta_cls),
                                            _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta, dbeta_cls


def lot_cross_attention_bwd(Q, K, V, Z, beta, eps, iters, dO, mass_q=None, mass_k=None, workspace=None,
                            path=PATH_AUTO):
    """(dQ, dK, dV, dZ, dbeta) of <lot_cross_attention_fwd(...), dO>; the masses are not differentiated."""
    B, H, n_q, n_k, d_k, d_v, r, code = _dims(Q, K, V, Z, beta, cross=True)
    _require(dO, "dO", Q.dtype, (B, H, n_q, d_v), Q.device)
    shape = lot_xshape(B, H, n_q, n_k, d_k, d_v, r, code)
    _masses(mass_q, mass_k, B, H, n_q, n_k, Q.device)
    workspace = _workspace(workspace, lot_cross_attention_bwd_workspace_bytes(shape, iters, path), Q.device)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    dZ, dbeta = torch.empty_like(Z), torch.empty_like(beta)
    _check(lib().lot_cross_attention_bwd_path(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Z), _ptr(beta),
                                              _ptr(mass_q), _ptr(mass_k),
                                              ctypes.c_float(eps), int(iters), _ptr(dO),
                                              _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(dZ), _ptr(dbeta),
                                              _ptr(workspace), ctypes.c_size_t(workspace.numel()), _stream(), int(path)))
    return dQ, dK, dV, dZ, dbeta


# ---------------------------------------------------------------------------------------------
# status of the waits between workgroups, testing aids, version
# ---------------------------------------------------------------------------------------------
def lot_workspace_status(workspace) -> int:
    """Synchronises the device and reads the status words of this workspace (0, or -10: a wait gave up)."""
    return lib().lot_workspace_status(_ptr(workspace))


class StatusProbe:
    """The status words of a workspace, copied to pinned host memory on the current stream without any
    synchronisation.  `ready()` says whether the stream has passed the copy; `failed()` waits for exactly
    that point (not for the device) and tells whether a wait between workgroups gave up in the last
    launch on that workspace.  The pinned words are taken from, and returned to, a small pool."""

    _pool = []

    def __init__(self, workspace):
        self.words = StatusProbe._pool.pop() if StatusProbe._pool else torch.zeros(2, dtype=torch.int64, pin_memory=True)
        _check(lib().lot_workspace_status_async(_ptr(workspace), ctypes.c_void_p(self.words.data_ptr()), _stream()))
        self.done = torch.cuda.Event()
        self.done.record()
        self._result = None

    def ready(self) -> bool:
        return self._result is not None or self.done.query()

    def failed(self) -> bool:
        if self._result is None:
            self.done.synchronize()
            self._result = lib().lot_status_words(ctypes.c_void_p(self.words.data_ptr())) == ERR_SYNC
            StatusProbe._pool.append(self.words)
            self.words = None
        return self._result


def lot_debug_set(knob: int, value: int) -> None:
    """Testing aid (see include/lot.h); value < 0 restores the default."""
    _check(lib().lot_debug_set(int(knob), int(value)))


def lot_version() -> int:
    return lib().lot_version()
