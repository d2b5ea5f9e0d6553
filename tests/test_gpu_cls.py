"""GPU parity of lot_attention_cls_fwd ([CLS] softmax row + LOT attention among the other tokens)
against the oracle, element by element; both execution paths; the DeiT shape at full size on
sampled problems.  Bars as for the plain forward: fp32 1e-4, bf16 I/O 2e-2 (max-norm relative)."""
import dataclasses

import numpy as np
import pytest

from paper_2509_23436_amd import synth
from util import rel_max_err, to_device, to_host_f64, tolerance

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


def S(w, **kw):
    return dataclasses.replace(w, **kw)


CASES = {
    "tiny": S(W["tiny"], n=65),
    "deit_like_f32": S(W["deit_tiny"], B=4, H=3, seed=80),                 # n = 197 = 196 + [CLS]
    "two_tokens": S(W["tiny"], n=2, r=1, seed=81),
    "bf16_ragged": S(W["long_4k"], B=2, H=2, n=1030, iters=5, seed=82),
    "bf16_d32": S(W["swin_t_s1"], B=2, H=3, n=400, seed=83),
    # 999 tokens among themselves, no more problems than compute units: four wavefronts per side
    "bf16_four_wavefronts_per_side": S(W["bert_base"], B=1, H=2, n=1000, r=32, iters=6, seed=86),
    "reference_only": S(W["tiny"], B=1, H=2, n=90, d=16, r=80, iters=4, seed=84),
    "several_softmax_chunks": S(W["tiny"], B=1, H=2, n=5000, d=32, r=8, iters=4, seed=85),
    "grouped_r128_bf16": S(W["long_4k"], B=1, H=2, n=700, r=128, iters=4, seed=87),   # 64 < r <= 256: grouped kernels
    # head widths below and above what one pass of the softmax row's lane groups covers (16 lanes x 4 columns)
    "narrow_head": S(W["tiny"], B=1, H=2, n=300, d=8, r=8, iters=4, seed=89),
    "wide_head": S(W["tiny"], B=1, H=2, n=261, d=136, r=8, iters=4, seed=90),
}


def _paths(w):
    fused = w.d in (32, 64) and w.r <= 256
    return ["reference", "fused"] if fused else ["reference"]


@pytest.mark.parametrize("name,path_name", [(nm, pn) for nm in CASES for pn in _paths(CASES[nm])])
def test_cls_variant_matches_oracle(name, path_name):
    import torch
    from oracle import lot_oracle
    from paper_2509_23436_amd import lot
    path = {"reference": lot.PATH_REFERENCE, "fused": lot.PATH_FUSED}[path_name]
    w = CASES[name]
    print("case %s path %s: %r" % (name, path_name, w), flush=True)
    x = synth.make_inputs(w)
    beta_cls = 0.9
    ref = lot_oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, beta_cls, threads=4)
    dev = to_device(x, w.dtype)
    out = lot.lot_attention_cls_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters, beta_cls,
                                    path=path)
    torch.cuda.synchronize()
    tol, _ = tolerance(w.dtype)
    O = to_host_f64(out)
    assert np.isfinite(O).all()
    err_cls = rel_max_err(O[:, :, 0], ref[:, :, 0])
    err_rest = rel_max_err(O[:, :, 1:], ref[:, :, 1:]) if w.n > 1 else 0.0
    print("  [CLS] row rel err %.3e, other rows rel err %.3e (bar %.0e)" % (err_cls, err_rest, tol), flush=True)
    assert err_cls <= tol and err_rest <= tol


def test_cls_variant_full_size_deit_on_sampled_problems():
    import torch
    from oracle import lot_oracle
    from paper_2509_23436_amd import lot
    w = W["deit_tiny"]
    x = synth.make_inputs(w)
    dev = to_device(x, w.dtype)
    out = lot.lot_attention_cls_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters, 1.0)
    torch.cuda.synchronize()
    O = to_host_f64(out).reshape(w.G, w.n, w.d)
    for gi in (0, 100, 191):
        b, h = gi // w.H, gi % w.H
        sl = lambda t: np.ascontiguousarray(t[b:b + 1, h:h + 1])           # noqa: E731
        ref = lot_oracle.attention_cls(sl(x["Q"]), sl(x["K"]), sl(x["V"]), x["Z"][h:h + 1], x["beta"][h:h + 1],
                                       w.eps, w.iters, 1.0)
        err = rel_max_err(O[gi], ref[0, 0])
        print("  problem %d rel err %.3e" % (gi, err), flush=True)
        assert err <= 1e-4


# ---- backward

BWD_CASES = {
    "tiny": S(W["tiny"], n=65),
    "deit_like_f32": S(W["deit_tiny"], B=2, H=3, iters=6, seed=86),
    "two_tokens": S(W["tiny"], n=2, r=1, seed=81),
    "bf16_ragged": S(W["long_4k"], B=1, H=2, n=1030, iters=5, seed=82),
    "bf16_d32": S(W["swin_t_s1"], B=2, H=3, n=400, seed=83),
    # 999 tokens among themselves, no more problems than compute units: four wavefronts per side
    "bf16_four_wavefronts_per_side": S(W["bert_base"], B=1, H=2, n=1000, r=32, iters=6, seed=86),
    "reference_only": S(W["tiny"], B=1, H=2, n=90, d=16, r=80, iters=4, seed=84),
    "several_softmax_chunks": S(W["tiny"], B=1, H=2, n=2600, d=32, r=8, iters=3, seed=85),
    # more than 64 pivots: the grouped tile kernels, here with the row stride of the [CLS] layout
    "grouped_r128_bf16": S(W["long_4k"], B=1, H=2, n=700, r=128, iters=4, seed=87),
    "grouped_r80_f32": S(W["tiny"], B=1, H=2, n=290, d=32, r=80, iters=4, seed=88),
    "narrow_head": S(W["tiny"], B=1, H=2, n=300, d=8, r=8, iters=4, seed=89),
    "wide_head": S(W["tiny"], B=1, H=2, n=261, d=136, r=8, iters=4, seed=90),
    "wide_head_bf16_chunks": S(W["long_4k"], B=1, H=1, n=2100, d=136, r=8, iters=3, seed=91),
}


def _bwd_paths(w):
    tiled = w.d in (32, 64) and w.r <= 64 and w.iters <= 64
    grouped = w.d in (32, 64) and 64 < w.r <= 256 and w.iters <= 64
    return ["reference", "fused"] if tiled or grouped else ["reference"]


@pytest.mark.parametrize("name,path_name", [(nm, pn) for nm in BWD_CASES for pn in _bwd_paths(BWD_CASES[nm])])
def test_cls_backward_matches_oracle(name, path_name):
    import torch
    from oracle import lot_oracle_bwd
    from paper_2509_23436_amd import lot
    path = {"reference": lot.PATH_REFERENCE, "fused": lot.PATH_FUSED}[path_name]
    w = BWD_CASES[name]
    print("case %s path %s: %r" % (name, path_name, w), flush=True)
    x = synth.make_inputs(w)
    dO = np.random.default_rng(w.seed + 17).standard_normal(x["V"].shape).astype(np.float32)
    if w.dtype == "bf16":
        dO = synth.round_to_bf16(dO)
    beta_cls = 0.9
    refs, _ = lot_oracle_bwd.attention_cls_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, beta_cls, dO)
    dev = to_device(dict(x, dO=dO), w.dtype)
    got = lot.lot_attention_cls_bwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters, beta_cls,
                                    dev["dO"], path=path)
    torch.cuda.synchronize()
    tol = 2e-2 if w.dtype == "bf16" else 1e-4
    for nm, g, ref in zip(("dQ", "dK", "dV", "dZ", "dbeta", "dbeta_cls"), got, refs):
        g = to_host_f64(g)
        assert np.isfinite(g).all(), nm
        scale = np.abs(ref).max()
        if scale < 1e-12:                       # identically zero (one pivot: nothing moves the plan)
            assert np.abs(g).max() <= 1e-6, nm
            continue
        err = rel_max_err(g, ref)
        print("  %-9s max-norm rel err %.3e (bar %.0e)" % (nm, err, tol), flush=True)
        assert err <= tol, nm
        if nm in ("dQ", "dK", "dV"):            # the [CLS] rows on their own scale
            err0 = rel_max_err(g[:, :, 0], ref[:, :, 0])
            print("  %-9s row 0 rel err %.3e" % (nm, err0), flush=True)
            assert err0 <= tol, nm


def test_cls_backward_full_size_deit_on_sampled_problems():
    import torch
    from oracle import lot_oracle_bwd
    from paper_2509_23436_amd import lot
    w = W["deit_tiny"]
    x = synth.make_inputs(w)
    dO = np.random.default_rng(9).standard_normal(x["V"].shape).astype(np.float32)
    dev = to_device(dict(x, dO=dO), w.dtype)
    got = lot.lot_attention_cls_bwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], w.eps, w.iters, 1.0, dev["dO"])
    torch.cuda.synchronize()
    for gi in (0, 191):
        b, h = gi // w.H, gi % w.H
        sl = lambda t: np.ascontiguousarray(t[b:b + 1, h:h + 1])           # noqa: E731
        refs, _ = lot_oracle_bwd.attention_cls_bwd(sl(x["Q"]), sl(x["K"]), sl(x["V"]), x["Z"][h:h + 1],
                                                   x["beta"][h:h + 1], w.eps, w.iters, 1.0, sl(dO))
        for nm, g, ref in zip(("dQ", "dK", "dV"), got[:3], refs[:3]):
            err = rel_max_err(to_host_f64(g[b:b + 1, h:h + 1]), ref)
            print("  problem %d %-5s rel err %.3e" % (gi, nm, err), flush=True)
            assert err <= 1e-4, nm
        err = abs(float(got[5][b, h]) - float(refs[5][0, 0])) / max(1e-12, abs(float(refs[5][0, 0])))
        print("  problem %d dbeta_cls rel err %.3e" % (gi, err), flush=True)
        assert err <= 1e-4


@pytest.mark.parametrize("d,d_v,bf16", [(16, 40, False), (24, 8, False), (72, 136, True)])
def test_cls_variant_with_value_width_other_than_key_width(d, d_v, bf16):
    """Forward and backward with d_v != d_k (plain kernels for the LOT part): the softmax row splits
    its threads by the key width for dq_cls and dK and by the value width for the output row and dV."""
    import torch
    from oracle import lot_oracle, lot_oracle_bwd
    from paper_2509_23436_amd import lot
    B, H, n, r, eps, iters, beta_cls = 1, 2, 150, 8, 0.1, 4, 1.3
    rng = np.random.default_rng(900 + d + d_v)
    x = {"Q": rng.standard_normal((B, H, n, d)) * d ** -0.5, "K": rng.standard_normal((B, H, n, d)) * d ** -0.5,
         "V": rng.standard_normal((B, H, n, d_v)), "Z": rng.standard_normal((H, r, d)) * d ** -0.5,
         "dO": rng.standard_normal((B, H, n, d_v))}
    x = {k: v.astype(np.float32) for k, v in x.items()}
    if bf16:
        x = {k: synth.round_to_bf16(v) for k, v in x.items()}
    b = rng.random((H, r)) + 0.2
    x["beta"] = (b / b.sum(axis=-1, keepdims=True)).astype(np.float32)
    print("case d=%d d_v=%d bf16=%s n=%d r=%d" % (d, d_v, bf16, n, r), flush=True)
    dtype = "bf16" if bf16 else "f32"
    tol = 2e-2 if bf16 else 1e-4
    dev = to_device(x, dtype)
    ref = lot_oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, beta_cls)
    out = lot.lot_attention_cls_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, beta_cls)
    torch.cuda.synchronize()
    O = to_host_f64(out)
    assert O.shape == ref.shape
    err = max(rel_max_err(O[:, :, 0], ref[:, :, 0]), rel_max_err(O[:, :, 1:], ref[:, :, 1:]))
    print("  forward rel err %.3e (bar %.0e)" % (err, tol), flush=True)
    assert err <= tol
    refs, _ = lot_oracle_bwd.attention_cls_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, beta_cls, x["dO"])
    got = lot.lot_attention_cls_bwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, beta_cls, dev["dO"])
    torch.cuda.synchronize()
    for nm, g, rf in zip(("dQ", "dK", "dV", "dZ", "dbeta", "dbeta_cls"), got, refs):
        g = to_host_f64(g)
        assert g.shape == rf.shape, nm
        e = rel_max_err(g, rf)
        print("  %-9s rel err %.3e" % (nm, e), flush=True)
        assert e <= tol, nm
        if nm in ("dQ", "dK", "dV"):
            assert rel_max_err(g[:, :, 0], rf[:, :, 0]) <= tol, nm
