"""lot_attention_fwd_static -- the forward for callers that cannot allocate: no workspace argument, the
scratch memory is a fixed array inside the library.  Through the C ABI, its output must equal that of
lot_attention_fwd (same kernels, caller-owned workspace) bit for bit and meet the oracle's bar, on two
calls in a row, the second with a smaller input (the array keeps what the first call left in it)."""
import dataclasses

import numpy as np
import pytest

from paper_2509_23436_amd import synth
from util import rel_max_err, to_device, to_host_f64, tolerance

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def _bits(t):
    import torch
    return t.view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32)


@pytest.mark.parametrize("first,second", [
    # several workgroups per problem (they exchange through the scratch array), then a smaller input
    (dataclasses.replace(W["long_4k"], B=1, H=2, n=4096, iters=6, seed=201),
     dataclasses.replace(W["long_4k"], B=1, H=2, n=1000, iters=4, seed=202)),
    # fp32 I/O, one workgroup per problem; then fewer, shorter problems
    (dataclasses.replace(W["deit_tiny"], B=8, iters=5, seed=203),
     dataclasses.replace(W["deit_tiny"], B=2, n=77, r=5, iters=7, seed=204)),
    # more than 64 pivots: the grouped kernels keep per-iteration tables in the scratch array
    (dataclasses.replace(W["long_4k"], B=1, H=2, n=3000, r=128, iters=5, seed=205),
     dataclasses.replace(W["long_4k"], B=1, H=1, n=500, r=100, iters=3, seed=206)),
])
def test_static_scratch_entry_point_matches_the_one_with_a_workspace(first, second):
    import torch
    from oracle import lot_oracle
    from paper_2509_23436_amd import lot
    assert lot.lot_static_scratch_bytes() == 32 << 20
    for w in (first, second):
        print("case %r" % (w,), flush=True)
        x = synth.make_inputs(w)
        dev = to_device(x, w.dtype)
        want = lot.lot_attention_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters)
        out = torch.full_like(dev["V"], float("nan"))
        lot.lot_attention_fwd_static(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters, out)
        torch.cuda.synchronize()
        assert torch.equal(_bits(out), _bits(want))
        O_ref, _ = lot_oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, threads=8)
        err = rel_max_err(to_host_f64(out), O_ref)
        print("  max-norm rel err against the oracle %.3e (bar %.0e)" % (err, tolerance(w.dtype)[0]), flush=True)
        assert err <= tolerance(w.dtype)[0]


def test_a_shape_beyond_the_fixed_array_is_refused_before_anything_runs():
    import ctypes
    import torch
    from paper_2509_23436_amd import lot
    # the plain kernels (d = 48 is outside the tile kernels' set) keep n x r intermediates: far beyond 32 MiB
    shape = lot.lot_shape(2, 8, 16384, 48, 48, 64, lot.LOT_F32)
    assert lot.lot_workspace_bytes(shape, 5) > lot.lot_static_scratch_bytes()
    vp = ctypes.c_void_p
    rc = lot.lib().lot_attention_fwd_static(ctypes.byref(shape), vp(4096), vp(8192), vp(12288), vp(256), vp(512),
                                            ctypes.c_float(0.1), 5, vp(16384), None)
    assert rc == -11
    assert b"scratch" in lot.lib().lot_strerror(rc)
    torch.cuda.synchronize()
