"""Host-only checks of the C ABI: the library loads, exports every declared symbol, and rejects bad
arguments before touching the device (so none of this needs a GPU)."""
import ctypes
import os
import re

import pytest

from paper_2509_23436_amd import lot

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lot.LIB_PATH):
        from paper_2509_23436_amd import build
        build.build()
    return lot.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "lot.h")).read()
    declared = set(re.findall(r"\b(lot_[a-z_]+)\s*\(", header))
    assert declared == set(lot.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name
    assert L.lot_version() >= 100


def _shape(**kw):
    base = dict(B=1, H=1, n=64, d_k=32, d_v=32, r=8, io_dtype=0)
    base.update(kw)
    return lot.lot_shape(**base)


def test_workspace_bytes_and_shape_validation(L):
    out = ctypes.c_size_t(0)
    assert L.lot_workspace_bytes(ctypes.byref(_shape()), 5, ctypes.byref(out)) == 0
    assert out.value > 0 and out.value % 256 == 0
    big = ctypes.c_size_t(0)
    assert L.lot_workspace_bytes(ctypes.byref(_shape(n=4096)), 5, ctypes.byref(big)) == 0
    assert big.value > out.value
    for bad in (dict(n=0), dict(r=0), dict(B=0), dict(H=-1), dict(d_k=0), dict(d_v=0), dict(n=1 << 25),
                dict(d_k=30), dict(d_v=6), dict(B=1 << 12, H=17)):
        assert L.lot_workspace_bytes(ctypes.byref(_shape(**bad)), 5, ctypes.byref(out)) == -2, bad
    assert L.lot_workspace_bytes(ctypes.byref(_shape(io_dtype=7)), 5, ctypes.byref(out)) == -5
    assert L.lot_workspace_bytes(ctypes.byref(_shape()), 0, ctypes.byref(out)) == -4
    assert L.lot_workspace_bytes(None, 5, ctypes.byref(out)) == -1
    assert L.lot_workspace_bytes(ctypes.byref(_shape()), 5, None) == -1


def _need(fn, shape, iters, *path):
    out = ctypes.c_size_t(0)
    rc = fn(ctypes.byref(shape), iters, *path, ctypes.byref(out))
    assert rc == 0, rc
    return out.value


def test_workspace_is_sized_for_the_kernels_that_run(L):
    """The tile kernels keep nothing of size n x r, and the workspace query must say so: it returns what the
    kernels AUTO selects use; the plain kernels' n x r intermediates are charged only to a caller who
    forces them."""
    MB = 1 << 20
    headline = lot.lot_shape(2, 8, 16384, 64, 64, 64, lot.LOT_BF16)
    auto = _need(L.lot_workspace_bytes, headline, 10)
    assert auto <= 32 * MB
    assert auto == _need(L.lot_workspace_bytes_path, headline, 10, lot.PATH_AUTO)
    assert auto == _need(L.lot_workspace_bytes_path, headline, 10, lot.PATH_FUSED)
    assert auto == _need(L.lot_couplings_workspace_bytes, headline, 10, lot.PATH_AUTO)
    plain = _need(L.lot_workspace_bytes_path, headline, 10, lot.PATH_REFERENCE)
    assert plain >= 4 * 16 * 16384 * 64 * 4           # two similarity matrices and two couplings
    assert _need(L.lot_attention_bwd_workspace_bytes, headline, 10) <= 128 * MB    # per-iteration Gram matrices
    assert _need(L.lot_attention_bwd_workspace_bytes_path, headline, 10, lot.PATH_REFERENCE) >= 5 * 2 * 16 * 16384 * 64 * 4
    # the largest point of the paper's runtime grid (grouped kernels)
    corner = lot.lot_shape(1, 8, 131072, 64, 64, 256, lot.LOT_BF16)
    assert _need(L.lot_workspace_bytes, corner, 5) <= 64 * MB
    assert _need(L.lot_attention_bwd_workspace_bytes, corner, 5) <= 1024 * MB
    # lot_couplings has no grouped kernels: beyond 64 pivots it is the plain kernels under AUTO too
    assert _need(L.lot_couplings_workspace_bytes, corner, 5, lot.PATH_AUTO) > 1024 * MB
    out = ctypes.c_size_t(0)
    assert L.lot_couplings_workspace_bytes(ctypes.byref(corner), 5, lot.PATH_FUSED, ctypes.byref(out)) == -9
    assert L.lot_workspace_bytes_path(ctypes.byref(_shape(d_k=128, d_v=128)), 5, lot.PATH_FUSED, ctypes.byref(out)) == -9
    assert L.lot_workspace_bytes_path(ctypes.byref(_shape()), 5, 9, ctypes.byref(out)) == -9
    # the backward of short or two-pivot fp32 problems runs on the plain kernels under AUTO
    short = _shape(n=12)
    assert _need(L.lot_attention_bwd_workspace_bytes, short, 5) == \
        _need(L.lot_attention_bwd_workspace_bytes_path, short, 5, lot.PATH_REFERENCE)
    two = _shape(n=4096, r=2)
    assert _need(L.lot_attention_bwd_workspace_bytes, two, 5) == \
        _need(L.lot_attention_bwd_workspace_bytes_path, two, 5, lot.PATH_REFERENCE)
    # the path without waits between workgroups: the grouped kernels' few megabytes at any r <= 256, the same
    # backward workspace as the tile kernels otherwise use; not for lot_couplings, not outside d in {32, 64}
    assert _need(L.lot_workspace_bytes_path, headline, 10, lot.PATH_STEPWISE) <= 32 * MB
    assert _need(L.lot_workspace_bytes_path, corner, 5, lot.PATH_STEPWISE) == _need(L.lot_workspace_bytes, corner, 5)
    assert _need(L.lot_attention_bwd_workspace_bytes_path, headline, 10, lot.PATH_STEPWISE) == \
        _need(L.lot_attention_bwd_workspace_bytes, headline, 10)
    assert L.lot_couplings_workspace_bytes(ctypes.byref(headline), 10, lot.PATH_STEPWISE, ctypes.byref(out)) == -9
    assert L.lot_workspace_bytes_path(ctypes.byref(_shape(d_k=128, d_v=128)), 5, lot.PATH_STEPWISE, ctypes.byref(out)) == -9
    assert L.lot_workspace_bytes_path(ctypes.byref(_shape(r=300)), 5, lot.PATH_STEPWISE, ctypes.byref(out)) == -9
    # cross attention
    x = lot.lot_xshape(2, 8, 16384, 4096, 64, 64, 64, lot.LOT_BF16)
    assert _need(L.lot_cross_workspace_bytes, x, 10) <= 32 * MB
    assert _need(L.lot_cross_workspace_bytes_path, x, 10, lot.PATH_REFERENCE) > 64 * MB
    assert _need(L.lot_cross_attention_bwd_workspace_bytes, x, 10) <= 128 * MB


def test_a_call_checks_the_workspace_against_the_path_it_takes(L):
    headline = lot.lot_shape(2, 8, 16384, 64, 64, 64, lot.LOT_BF16)
    auto = _need(L.lot_workspace_bytes, headline, 10)
    assert _call_fwd(L, shape=headline, iters=10, ws_bytes=auto - 1) == -6
    assert _call_fwd(L, shape=headline, iters=10, ws_bytes=auto, path=lot.PATH_REFERENCE) == -6


def test_status_words_and_testing_knobs(L):
    words = (ctypes.c_ulonglong * 2)(0, 0)
    assert L.lot_status_words(words) == 0
    words[0], words[1] = 5, 7
    assert L.lot_status_words(words) == 0            # the failed launch is not the last one
    words[0] = 7
    assert L.lot_status_words(words) == -10
    assert L.lot_status_words(None) == -1
    assert L.lot_workspace_status_async(None, words, None) == -1
    assert L.lot_workspace_status_async(ctypes.c_void_p(4096), None, None) == -1
    assert L.lot_debug_set(lot.KNOB_SPIN_LIMIT, 0) == 0
    assert L.lot_debug_set(lot.KNOB_SPIN_LIMIT, -1) == 0
    assert L.lot_debug_set(17, 1) == -2 and L.lot_debug_set(-1, 1) == -2


def test_the_binding_checks_every_tensor_against_the_shape_before_calling(L):
    """The C ABI sees only pointers: a tensor that is shorter than the shape says would be read or
    written past its end.  The binding therefore compares every tensor with the others on the host."""
    import torch
    B, H, n, d, r = 2, 3, 40, 32, 8
    t = lambda *shape, dtype=torch.float32: torch.zeros(shape, dtype=dtype)      # noqa: E731
    good = dict(Q=t(B, H, n, d), K=t(B, H, n, d), V=t(B, H, n, d), Z=t(H, r, d), beta=t(H, r))

    def fwd(**kw):
        a = dict(good, **kw)
        return lot.lot_attention_fwd(a["Q"], a["K"], a["V"], a["Z"], a["beta"], 0.1, 3, out=a.get("out"))

    for kw in (dict(K=t(B, H, n - 1, d)), dict(K=t(B, H + 1, n, d)), dict(K=t(B, H, n, d + 8)), dict(V=t(B, H, n + 5, d)),
               dict(V=t(B + 1, H, n, d)), dict(Z=t(H, r, d + 32)), dict(Z=t(H - 1, r, d)), dict(beta=t(H, r + 1)),
               dict(beta=t(H * r)), dict(out=t(B, H, n - 1, d)), dict(out=t(B, H, n, 2 * d)),
               dict(Q=t(B * H, n, d)), dict(Q=t(B, H, n, d).transpose(2, 3))):
        with pytest.raises(ValueError):
            fwd(**kw)
    for kw in (dict(K=t(B, H, n, d, dtype=torch.bfloat16)), dict(Z=t(H, r, d, dtype=torch.bfloat16)),
               dict(beta=t(H, r, dtype=torch.float64)), dict(Q=t(B, H, n, d, dtype=torch.float16)),
               dict(out=t(B, H, n, d, dtype=torch.bfloat16))):
        with pytest.raises(TypeError):
            fwd(**kw)
    # consistent shapes on the host side: refused too (there is no CPU path), again before any call
    with pytest.raises(ValueError, match="device"):
        fwd()
    with pytest.raises(ValueError):
        lot.lot_couplings(good["Q"], t(B, H, n + 1, d), good["Z"], good["beta"], 0.1, 3)
    with pytest.raises(ValueError):
        lot.lot_attention_bwd(good["Q"], good["K"], good["V"], good["Z"], good["beta"], 0.1, 3, t(B, H, n, d + 8))
    with pytest.raises(ValueError):
        lot.lot_attention_cls_bwd(good["Q"], good["K"], good["V"], good["Z"], good["beta"], 0.1, 3, 1.0, t(B, H, n - 1, d))
    with pytest.raises(ValueError):     # cross attention: K and V must agree on the key count
        lot.lot_cross_attention_fwd(good["Q"], t(B, H, 70, d), t(B, H, 71, d), good["Z"], good["beta"], 0.1, 3)
    with pytest.raises(ValueError):
        lot.lot_cross_attention_fwd(good["Q"], t(B, H, 70, d), t(B, H, 70, d), good["Z"], good["beta"], 0.1, 3,
                                    mass_k=t(B, H, 69))
    with pytest.raises(ValueError):
        lot.lot_cross_attention_bwd(good["Q"], t(B, H, 70, d), t(B, H, 70, d), good["Z"], good["beta"], 0.1, 3,
                                    t(B, H, 70, d))     # dO must follow the queries


def _call_fwd(L, shape=None, Q=4096, K=8192, V=12288, Z=256, beta=512, eps=0.1, iters=5, out=16384,
              ws=1 << 20, ws_bytes=1 << 40, path=0):
    shape = shape or _shape()
    vp = ctypes.c_void_p
    return L.lot_attention_fwd_path(ctypes.byref(shape), vp(Q), vp(K), vp(V), vp(Z), vp(beta), ctypes.c_float(eps),
                                    iters, vp(out), vp(ws), ctypes.c_size_t(ws_bytes), None, path)


def test_attention_rejects_bad_arguments_before_any_device_work(L):
    # the pointers are fake: every one of these must return before they are used
    for kw, code in ((dict(Q=0), -1), (dict(K=0), -1), (dict(V=0), -1), (dict(Z=0), -1), (dict(beta=0), -1),
                     (dict(out=0), -1), (dict(ws=0), -1),
                     (dict(eps=0.0), -3), (dict(eps=-1.0), -3), (dict(eps=float("nan")), -3),
                     (dict(eps=float("inf")), -3), (dict(iters=0), -4),
                     (dict(Q=4100), -7), (dict(V=12290), -7), (dict(out=16388), -7),
                     (dict(ws=(1 << 20) + 64), -6), (dict(ws_bytes=1024), -6),
                     (dict(path=9), -9), (dict(shape=_shape(d_k=128, d_v=128), path=2), -9),
                     (dict(shape=_shape(r=257), path=2), -9),
                     (dict(shape=_shape(n=0)), -2), (dict(shape=_shape(io_dtype=3)), -5)):
        assert _call_fwd(L, **kw) == code, (kw, code)


def test_couplings_rejects_bad_arguments(L):
    vp = ctypes.c_void_p
    s = _shape()

    def call(g1=4096, g2=8192, eps=0.1, iters=3, ws_bytes=1 << 40):
        return L.lot_couplings(ctypes.byref(s), vp(256), vp(512), vp(1024), vp(2048), ctypes.c_float(eps), iters,
                               vp(g1), vp(g2), vp(1 << 20), ctypes.c_size_t(ws_bytes), None)
    assert call(g1=0) == -1 and call(g2=0) == -1
    assert call(eps=0.0) == -3 and call(iters=-2) == -4 and call(ws_bytes=0) == -6


def test_strerror_texts(L):
    for code in range(0, -12, -1):
        if code == -8:
            continue
        text = L.lot_strerror(code).decode()
        assert text and text != "unknown status"
    assert L.lot_strerror(-99).decode() == "unknown status"


def test_backward_rejects_bad_arguments(L):
    vp = ctypes.c_void_p
    s = _shape()
    need = ctypes.c_size_t(0)
    assert L.lot_attention_bwd_workspace_bytes(ctypes.byref(s), 5, ctypes.byref(need)) == 0
    fwd = ctypes.c_size_t(0)
    assert L.lot_workspace_bytes(ctypes.byref(s), 5, ctypes.byref(fwd)) == 0
    assert need.value > 0 and need.value % 256 == 0
    assert L.lot_attention_bwd_workspace_bytes(ctypes.byref(s), 0, ctypes.byref(need)) == -4
    assert L.lot_attention_bwd_workspace_bytes(ctypes.byref(s), 1 << 17, ctypes.byref(need)) == -4

    def call(dO=0x5000, dQ=0x6000, dZ=0x7000, eps=0.1, iters=5, ws=1 << 20, ws_bytes=1 << 40, path=0, shape=s):
        return L.lot_attention_bwd_path(ctypes.byref(shape), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x100), vp(0x200),
                                        ctypes.c_float(eps), iters, vp(dO), vp(dQ), vp(0x8000), vp(0x9000), vp(dZ),
                                        vp(0xA000), vp(ws), ctypes.c_size_t(ws_bytes), None, path)

    for kw, code in ((dict(dO=0), -1), (dict(dQ=0), -1), (dict(dZ=0), -1), (dict(ws=0), -1),
                     (dict(eps=0.0), -3), (dict(iters=0), -4), (dict(dO=0x5004), -7), (dict(dZ=0x7002), -7),
                     (dict(ws=(1 << 20) + 8), -6), (dict(ws_bytes=64), -6), (dict(path=5), -9),
                     (dict(path=2, shape=_shape(r=300)), -9), (dict(path=2, shape=_shape(d_k=48, d_v=48)), -9),
                     (dict(path=2, iters=65), -9),       # the tile kernels' per-iteration tables: 64 iterations at most
                     (dict(path=2, iters=65, shape=_shape(r=200, d_k=64, d_v=64)), -9)):
        assert call(**kw) == code, (kw, code)


def test_cls_and_cross_entry_points_reject_bad_arguments(L):
    vp = ctypes.c_void_p
    s = _shape()

    def cls(beta_cls=1.0, shape=s, out=0x4000):
        return L.lot_attention_cls_fwd(ctypes.byref(shape), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x100), vp(0x200),
                                       ctypes.c_float(0.1), 5, ctypes.c_float(beta_cls), vp(out), vp(1 << 20),
                                       ctypes.c_size_t(1 << 40), None)

    assert cls(beta_cls=0.0) == -3 and cls(beta_cls=float("nan")) == -3
    assert cls(shape=_shape(n=1)) == -2
    assert cls(out=0) == -1

    def cls_bwd(beta_cls=1.0, shape=s, dbc=0x8000, dO=0x5000, ws_bytes=1 << 40, eps=0.1):
        return L.lot_attention_cls_bwd(ctypes.byref(shape), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x100), vp(0x200),
                                       ctypes.c_float(eps), 5, ctypes.c_float(beta_cls), vp(dO),
                                       vp(0x6000), vp(0x7000), vp(0x9000), vp(0x300), vp(0x400), vp(dbc), vp(1 << 20),
                                       ctypes.c_size_t(ws_bytes), None)

    assert cls_bwd(beta_cls=-1.0) == -3 and cls_bwd(shape=_shape(n=1)) == -2
    assert cls_bwd(dbc=0) == -1 and cls_bwd(dO=0) == -1 and cls_bwd(dbc=0x8002) == -7
    assert cls_bwd(ws_bytes=64) == -6 and cls_bwd(eps=0.0) == -3

    x = lot.lot_xshape(1, 1, 40, 70, 32, 32, 8, 0)
    need = ctypes.c_size_t(0)
    assert L.lot_cross_workspace_bytes(ctypes.byref(x), 5, ctypes.byref(need)) == 0 and need.value % 256 == 0
    assert L.lot_cross_workspace_bytes(ctypes.byref(lot.lot_xshape(1, 1, 0, 70, 32, 32, 8, 0)), 5, ctypes.byref(need)) == -2
    assert L.lot_cross_workspace_bytes(ctypes.byref(lot.lot_xshape(1, 1, 40, 0, 32, 32, 8, 0)), 5, ctypes.byref(need)) == -2

    def cross(mq=0x5000, K=0x2000, eps=0.1, ws_bytes=1 << 40, path=0, shape=x):
        return L.lot_cross_attention_fwd_path(ctypes.byref(shape), vp(0x1000), vp(K), vp(0x3000), vp(0x100), vp(0x200),
                                              vp(mq), vp(0), ctypes.c_float(eps), 5, vp(0x4000), vp(1 << 20),
                                              ctypes.c_size_t(ws_bytes), None, path)

    for kw, code in ((dict(K=0), -1), (dict(eps=-1.0), -3), (dict(mq=0x5002), -7), (dict(ws_bytes=128), -6),
                     (dict(path=7), -9), (dict(path=2, shape=lot.lot_xshape(1, 1, 40, 70, 16, 16, 8, 0)), -9)):
        assert cross(**kw) == code, (kw, code)

    def cross_bwd(mq=0x5000, dO=0x6000, eps=0.1, ws_bytes=1 << 40, iters=5, shape=x, dQ=0x7000):
        return L.lot_cross_attention_bwd(ctypes.byref(shape), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x100), vp(0x200),
                                         vp(mq), vp(0), ctypes.c_float(eps), iters, vp(dO), vp(dQ), vp(0x8000), vp(0x9000),
                                         vp(0x300), vp(0x400), vp(1 << 20), ctypes.c_size_t(ws_bytes), None)

    assert L.lot_cross_attention_bwd_workspace_bytes(ctypes.byref(x), 5, ctypes.byref(need)) == 0 and need.value % 256 == 0
    assert L.lot_cross_attention_bwd_workspace_bytes(ctypes.byref(x), 0, ctypes.byref(need)) == -4
    for kw, code in ((dict(dO=0), -1), (dict(dQ=0), -1), (dict(eps=0.0), -3), (dict(iters=0), -4), (dict(mq=0x5002), -7),
                     (dict(dO=0x6004), -7), (dict(ws_bytes=128), -6),
                     (dict(shape=lot.lot_xshape(1, 1, 40, 0, 32, 32, 8, 0)), -2)):
        assert cross_bwd(**kw) == code, (kw, code)
