"""Seeded synthetic inputs for LOT attention (inputs only: none of the method's arithmetic).

Both the CPU oracle's tests and the HIP path's tests draw their inputs from here, so that the
two sides see identical bits on any machine.  The generator is counter based (a splitmix64
hash of seed, stream and element index, then Box-Muller), so any element can be produced
without generating the ones before it and the result does not depend on numpy's own
random-number streams.

Recipe (the paper's workloads, shapes only): Q, K, V, Z are i.i.d. N(0,1) scaled by d^-1/2;
the pivot masses (the paper's p^0 / sigma, "Empirical measures and pivot" in Method) are the
softmax of r i.i.d. N(0,1) logits per head, hence strictly positive and summing to one.  For
the bf16 workloads Q, K, V and (by default) Z are rounded to bf16 (round to nearest even) here,
before either side reads them, so input rounding is not part of any error that is compared.  The
library takes Z in fp32 whatever the I/O type (a learnable parameter): `round_pivots=False` leaves it
unrounded, so that the library's own handling of an ordinary fp32 Z is compared as well.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# stream ids: one per tensor, in the order Q, K, V, Z, logits
STREAM_Q, STREAM_K, STREAM_V, STREAM_Z, STREAM_LOGITS = 0, 1, 2, 3, 4


def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _M1
        x = (x ^ (x >> np.uint64(27))) * _M2
        x = x ^ (x >> np.uint64(31))
    return x


def standard_normal(seed: int, stream: int, shape) -> np.ndarray:
    """N(0,1) doubles by Box-Muller from two counter-based uniform words per element."""
    count = int(np.prod(shape)) if len(shape) else 1
    out = np.empty(count, dtype=np.float64)
    step = 1 << 22                                   # bound the temporaries
    for lo in range(0, count, step):
        hi = min(count, lo + step)
        with np.errstate(over="ignore"):
            key0 = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]) * _GAMMA
                          + np.uint64(stream * 2 + 1))
            key1 = _mix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]) * _GAMMA
                          + np.uint64(stream * 2 + 2))
            idx = np.arange(lo + 1, hi + 1, dtype=np.uint64) * _GAMMA
            w0 = _mix64(key0 + idx)
            w1 = _mix64(key1 + idx)
        # 53-bit uniforms; u0 in (0,1] so the log is finite
        u0 = ((w0 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        u1 = (w1 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[lo:hi] = np.sqrt(-2.0 * np.log(u0)) * np.cos(2.0 * np.pi * u1)
        del w0, w1, u0, u1, idx
    return out.reshape(shape)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array whose values are exactly representable in bf16 (round to nearest even)."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((bits >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        rounded = (bits + bias) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The upper 16 bits (uint16) of float32 values that are already bf16 representable."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(bits & np.uint32(0xFFFF)), "values are not bf16 representable"
    return (bits >> np.uint32(16)).astype(np.uint16)


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    n: int
    d: int          # d_k = d_v
    r: int
    dtype: str      # "f32" or "bf16": dtype of Q, K, V and of the output
    eps: float
    iters: int
    seed: int

    @property
    def G(self) -> int:
        return self.B * self.H

    @property
    def tokens(self) -> int:            # sequence tokens per call
        return self.B * self.n


# The five workload shapes (DeiT-Tiny, BERT-base, Swin-T stage 1, long context) plus the tiny case.
WORKLOADS = {
    "tiny":       Workload("tiny", 1, 1, 64, 32, 8, "f32", 0.1, 20, 0),
    "deit_tiny":  Workload("deit_tiny", 64, 3, 197, 64, 16, "f32", 0.1, 10, 2),
    "bert_base":  Workload("bert_base", 32, 12, 512, 64, 32, "bf16", 0.05, 10, 3),
    "swin_t_s1":  Workload("swin_t_s1", 16, 3, 3136, 32, 32, "bf16", 0.1, 10, 4),
    "long_4k":    Workload("long_4k", 2, 8, 4096, 64, 64, "bf16", 0.05, 10, 50),
    "long_16k":   Workload("long_16k", 2, 8, 16384, 64, 64, "bf16", 0.05, 10, 51),
    "long_64k":   Workload("long_64k", 2, 8, 65536, 64, 64, "bf16", 0.05, 10, 52),
}


def shrink(w: Workload, **kw) -> Workload:
    return replace(w, **kw)


def make_inputs(w: Workload, d_v: int | None = None, round_pivots: bool = True) -> dict:
    """Q, K: [B,H,n,d]; V: [B,H,n,d_v]; Z: [H,r,d]; beta: [H,r] -- all float32 numpy arrays.

    For dtype == "bf16" the values of Q, K, V (and of Z unless round_pivots is False) are bf16
    representable (see `bf16_bits`).
    """
    d_v = w.d if d_v is None else d_v
    scale = float(w.d) ** -0.5
    q = (standard_normal(w.seed, STREAM_Q, (w.B, w.H, w.n, w.d)) * scale).astype(np.float32)
    k = (standard_normal(w.seed, STREAM_K, (w.B, w.H, w.n, w.d)) * scale).astype(np.float32)
    v = (standard_normal(w.seed, STREAM_V, (w.B, w.H, w.n, d_v)) * scale).astype(np.float32)
    z = (standard_normal(w.seed, STREAM_Z, (w.H, w.r, w.d)) * scale).astype(np.float32)
    logits = standard_normal(w.seed, STREAM_LOGITS, (w.H, w.r))
    e = np.exp(logits - logits.max(axis=1, keepdims=True))
    beta = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    if w.dtype == "bf16":
        q, k, v = (round_to_bf16(t) for t in (q, k, v))
        if round_pivots:
            z = round_to_bf16(z)
    return {"Q": q, "K": k, "V": v, "Z": z, "beta": beta}


def to_device(x: dict, dtype: str) -> dict:
    """numpy inputs (float32; Q, K, V, dO bf16-representable when dtype == 'bf16') -> torch device tensors.
    Z and beta stay float32 whatever the I/O type."""
    import torch
    dev = {}
    for k in ("Q", "K", "V", "dO"):
        if k not in x:
            continue
        if dtype == "bf16":
            bits = bf16_bits(x[k]).view(np.int16)
            dev[k] = torch.from_numpy(bits).cuda().view(torch.bfloat16)
        else:
            dev[k] = torch.from_numpy(np.ascontiguousarray(x[k])).cuda()
    dev["Z"] = torch.from_numpy(np.ascontiguousarray(x["Z"], dtype=np.float32)).cuda()
    dev["beta"] = torch.from_numpy(np.ascontiguousarray(x["beta"], dtype=np.float32)).cuda()
    return dev
