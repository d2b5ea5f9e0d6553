"""Pins of the backward oracle (oracle/lot_oracle_bwd.py) to things other than itself.

The paper prints no worked example of a gradient, so the pins are: the C oracle's forward (a
different implementation, different language), central finite differences of that forward, and
closed forms that follow from the method's structure.
"""
import dataclasses

import numpy as np
import pytest

from paper_2509_23436_amd import synth

W = synth.WORKLOADS


def _case(B=2, H=2, n=24, d=8, r=5, eps=0.1, iters=4, seed=900, d_v=None):
    w = dataclasses.replace(W["tiny"], B=B, H=H, n=n, d=d, r=r, eps=eps, iters=iters, seed=seed, dtype="f32")
    x = synth.make_inputs(w, d_v=d_v)
    x = {k: np.asarray(v, dtype=np.float64) for k, v in x.items()}
    rng = np.random.default_rng(seed + 1)
    dO = rng.standard_normal(x["V"].shape)
    return w, x, dO


def _loss_c(oracle, x, w, dO):
    O, _ = oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, threads=2)
    return float((O * dO).sum())


def test_forward_of_the_backward_oracle_equals_the_c_oracle(oracle):
    from oracle import lot_oracle_bwd
    for kw in (dict(), dict(r=1), dict(n=33, r=7, iters=7, eps=0.05), dict(d_v=12)):
        w, x, dO = _case(**kw)
        _, O_t = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, dO)
        O_c, _ = oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters, threads=2)
        assert np.abs(O_t - O_c).max() <= 1e-12 * max(1.0, np.abs(O_c).max())


@pytest.mark.parametrize("kw", [dict(), dict(eps=0.05, iters=6, n=17, r=4), dict(iters=1), dict(d_v=6, r=3)])
def test_gradients_match_central_differences_of_the_c_oracle(oracle, kw):
    # d/dh L(x + h v) at h = 0 for random directions v, one tensor at a time; L = <O, dO>.
    from oracle import lot_oracle_bwd
    w, x, dO = _case(**kw)
    (dQ, dK, dV, dZ, dbeta), _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"],
                                                              w.eps, w.iters, dO)
    grads = {"Q": dQ, "K": dK, "V": dV, "Z": dZ, "beta": dbeta}
    rng = np.random.default_rng(5)
    for name, g in grads.items():
        for _ in range(3):
            v = rng.standard_normal(x[name].shape)
            if name == "beta":
                v *= 0.1 * x["beta"]          # stays strictly positive
            h = 1e-6
            xp = dict(x); xm = dict(x)
            xp[name] = x[name] + h * v
            xm[name] = x[name] - h * v
            fd = (_loss_c(oracle, xp, w, dO) - _loss_c(oracle, xm, w, dO)) / (2 * h)
            an = float((g * v).sum())
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(an), abs(fd)), (name, fd, an)


def test_one_pivot_gives_the_mean_and_nothing_else_moves(oracle):
    # r = 1: Gamma1 = Gamma2^T = beta_1/n in every entry whatever Q, K, z, eps are, so
    # O_i = beta_1 * mean(V) for every i.  Hence dV_j = (beta_1/n) sum_i dO_i for every j,
    # dbeta_1 = sum_i <dO_i, mean(V)> (summed over the batch), and dQ = dK = dZ = 0.
    from oracle import lot_oracle_bwd
    w, x, dO = _case(r=1, n=19, iters=3)
    x["beta"] = x["beta"] * np.array([[0.7], [1.3]])          # masses need not sum to one for this identity
    (dQ, dK, dV, dZ, dbeta), _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"],
                                                              w.eps, w.iters, dO)
    b = x["beta"][None, :, :, None]                            # [1,H,1,1]
    want = np.broadcast_to(b * dO.mean(axis=2, keepdims=True), dV.shape)
    assert np.abs(dV - want).max() <= 1e-13
    want_b = (dO.sum(axis=2) * x["V"].mean(axis=2)).sum(axis=(0, 2))      # [H]
    assert np.abs(dbeta[:, 0] - want_b).max() <= 1e-12
    for g in (dQ, dK, dZ):
        assert np.abs(g).max() <= 1e-12


def test_common_shift_of_the_pivots_has_zero_gradient(oracle):
    # z_t -> z_t + v for all t adds a per-token constant to every similarity row, which the first
    # token-side update absorbs: no coupling changes, hence sum_t dZ_t = 0 for every head.
    from oracle import lot_oracle_bwd
    w, x, dO = _case(n=21, r=6, iters=5)
    (_, _, _, dZ, _), _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"],
                                                        w.eps, w.iters, dO)
    assert np.abs(dZ.sum(axis=1)).max() <= 1e-11 * max(1.0, np.abs(dZ).max())
    assert np.abs(dZ).max() > 1e-6      # the individual gradients are not trivially zero


def test_value_gradient_is_the_transposed_dense_plan(oracle):
    # O = A V with A = n P (dense n x n plan from the C oracle), so dV = A^T dO.
    from oracle import lot_oracle_bwd
    w, x, dO = _case(B=1, H=2, n=16, r=4, iters=5)
    (_, _, dV, _, _), _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"],
                                                        w.eps, w.iters, dO)
    for h in range(2):
        g1, g2 = oracle.couplings_one(x["Q"][0, h], x["K"][0, h], x["Z"][h], x["beta"][h], w.eps, w.iters)
        A = w.n * oracle.dense_plan(g1, g2, x["beta"][h])
        assert np.abs(dV[0, h] - A.T @ dO[0, h]).max() <= 1e-12
