"""Pins of the [CLS]-hybrid oracle (oracle.lot_oracle.attention_cls) to things other than itself."""
import dataclasses

import numpy as np
import scipy.special

from paper_2509_23436_amd import synth

W = synth.WORKLOADS


def _case(n=23, r=5, seed=300, **kw):
    w = dataclasses.replace(W["tiny"], B=2, H=2, n=n, d=8, r=r, iters=6, seed=seed, dtype="f32", **kw)
    x = {k: np.asarray(v, dtype=np.float64) for k, v in synth.make_inputs(w).items()}
    return w, x


def test_cls_row_is_the_library_softmax(oracle):
    w, x = _case()
    out = oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, 0.7)
    scores = 0.7 * np.einsum("bhc,bhjc->bhj", x["Q"][:, :, 0], x["K"])
    want = np.einsum("bhj,bhjc->bhc", scipy.special.softmax(scores, axis=-1), x["V"])
    assert np.abs(out[:, :, 0] - want).max() <= 1e-14


def test_cls_row_limits(oracle):
    w, x = _case()
    flat = oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, 1e-13)
    assert np.abs(flat[:, :, 0] - x["V"].mean(axis=2)).max() <= 1e-12          # temperature -> 0: plain mean
    sharp = oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, 1e6)
    best = np.einsum("bhc,bhjc->bhj", x["Q"][:, :, 0], x["K"]).argmax(axis=-1)
    for b in range(2):
        for h in range(2):
            assert np.abs(sharp[b, h, 0] - x["V"][b, h, best[b, h]]).max() <= 1e-9   # -> the best-matching key's value


def test_other_rows_are_the_plain_method_on_the_other_tokens_and_ignore_cls(oracle):
    w, x = _case()
    out = oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, 0.7)
    inner, _ = oracle.attention(x["Q"][:, :, 1:], x["K"][:, :, 1:], x["V"][:, :, 1:], x["Z"], x["beta"], w.eps, w.iters)
    assert np.array_equal(out[:, :, 1:], inner)
    y = {k: v.copy() for k, v in x.items()}
    for k in ("Q", "K", "V"):
        y[k][:, :, 0] += 3.0                                                       # a different [CLS] token
    out2 = oracle.attention_cls(y["Q"], y["K"], y["V"], y["Z"], y["beta"], w.eps, w.iters, 0.7)
    assert np.array_equal(out2[:, :, 1:], out[:, :, 1:])
    assert np.abs(out2[:, :, 0] - out[:, :, 0]).max() > 1e-3


def test_rows_of_the_hybrid_attention_matrix_sum_to_one(oracle):
    # Feeding V = identity (d_v = n) returns the attention matrix itself: every row sums to one, the
    # [CLS] column of the other rows is zero, and the block among the other tokens has unit column sums
    # once the solves have converged (doubly stochastic among the image tokens).
    n = 12
    w, x = _case(n=n, r=4, seed=301)
    x["beta"] = x["beta"] / x["beta"].sum(axis=-1, keepdims=True)     # float32 masses sum to one only to 1e-8
    eye = np.broadcast_to(np.eye(n), (2, 2, n, n)).copy()
    A = oracle.attention_cls(x["Q"], x["K"], eye, x["Z"], x["beta"], w.eps, 4000, 0.7)
    assert np.abs(A.sum(axis=-1) - 1.0).max() <= 1e-10
    assert np.abs(A[:, :, 1:, 0]).max() == 0.0
    assert np.abs(A[:, :, 1:, 1:].sum(axis=-2) - 1.0).max() <= 1e-9
