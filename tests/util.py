"""Helpers shared by the GPU tests: move seeded inputs to the device, run the oracle, compare."""
import numpy as np

from paper_2509_23436_amd import synth


def to_device(x, dtype):
    """numpy inputs (float32, bf16-representable when dtype == 'bf16') -> torch device tensors."""
    import torch
    dev = {}
    for k in ("Q", "K", "V", "dO"):
        if k not in x:
            continue
        if dtype == "bf16":
            bits = synth.bf16_bits(x[k]).view(np.int16)
            dev[k] = torch.from_numpy(bits).cuda().view(torch.bfloat16)
        else:
            dev[k] = torch.from_numpy(np.ascontiguousarray(x[k])).cuda()
    dev["Z"] = torch.from_numpy(np.ascontiguousarray(x["Z"])).cuda()
    dev["beta"] = torch.from_numpy(np.ascontiguousarray(x["beta"])).cuda()
    return dev


def to_host_f64(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel_max_err(got, ref):
    """max-norm relative error: max|got - ref| / max|ref| (the output has zero-mean entries, so an
    elementwise ratio is undefined)."""
    return float(np.abs(got - ref).max() / np.abs(ref).max())


def tolerance(dtype):
    """Bars stated for the target: fp32 <= 1e-4 on O and 1e-5 on marginals; bf16 I/O <= 2e-2 on O."""
    return (1e-4, 1e-5) if dtype == "f32" else (2e-2, 1e-5)
