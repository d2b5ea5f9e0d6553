"""Pins of the cross-attention / non-uniform-mass oracle (oracle.lot_oracle.cross_attention)."""
import dataclasses

import numpy as np

from paper_2509_23436_amd import synth

W = synth.WORKLOADS


def _case(n_q=20, n_k=31, r=5, d=8, d_v=6, seed=400, iters=6, eps=0.1):
    rng = np.random.default_rng(seed)
    B, H = 2, 2
    x = {"Q": rng.standard_normal((B, H, n_q, d)) * d ** -0.5, "K": rng.standard_normal((B, H, n_k, d)) * d ** -0.5,
         "V": rng.standard_normal((B, H, n_k, d_v)), "Z": rng.standard_normal((H, r, d)) * d ** -0.5}
    b = rng.random((H, r)) + 0.2
    x["beta"] = b / b.sum(axis=-1, keepdims=True)
    mq = rng.random((B, H, n_q)) + 0.1
    mk = rng.random((B, H, n_k)) + 0.1
    x["mq"] = mq / mq.sum(axis=-1, keepdims=True)
    x["mk"] = mk / mk.sum(axis=-1, keepdims=True)
    return x, eps, iters


def _run(oracle, x, eps, iters, **over):
    y = dict(x, **over)
    return oracle.cross_attention(y["Q"], y["K"], y["V"], y["Z"], y["beta"], y["mq"], y["mk"], eps, iters)


def test_uniform_masses_and_equal_lengths_give_the_plain_method(oracle):
    w = dataclasses.replace(W["tiny"], B=2, H=2, n=25, d=8, r=5, iters=5, seed=401, dtype="f32")
    x = {k: np.asarray(v, dtype=np.float64) for k, v in synth.make_inputs(w).items()}
    u = np.full((2, 2, 25), 1.0 / 25)
    got = oracle.cross_attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], u, u, w.eps, w.iters)
    want, _ = oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], w.eps, w.iters)
    assert np.abs(got - want).max() <= 1e-12


def test_rows_are_the_coupling_divided_by_the_mass(oracle):
    # for positive masses the row formula used by the oracle is Gamma1_it / mu_i with Gamma1 from the C pieces
    x, eps, iters = _case()
    eye = np.broadcast_to(np.eye(31), (2, 2, 31, 31)).copy()
    A = _run(oracle, x, eps, iters, V=eye)                               # the attention matrix itself
    for b in range(2):
        for h in range(2):
            C1 = oracle.cost(x["Q"][b, h], x["Z"][h]); C2 = oracle.cost(x["K"][b, h], x["Z"][h])
            f1, g1 = oracle.sinkhorn(C1, x["mq"][b, h], x["beta"][h], eps, iters)
            f2, g2 = oracle.sinkhorn(C2, x["mk"][b, h], x["beta"][h], eps, iters)
            G1 = oracle.coupling(C1, f1, g1, eps); G2 = oracle.coupling(C2, f2, g2, eps)
            glued = G1 @ np.diag(1.0 / x["beta"][h]) @ G2.T               # n_q x n_k plan between mu and nu
            assert np.abs(A[b, h] - glued / x["mq"][b, h][:, None]).max() <= 1e-12


def test_marginals_of_the_plan(oracle):
    # At every T the pivot side is exact in both solves (it is updated last), so the glued plan
    # Diag(mu) A has total mass one and its column sums are those of Gamma2; once the solves have
    # converged, rows of A sum to one and mu^T A = nu.
    x, eps, _ = _case()
    eye = np.broadcast_to(np.eye(31), (2, 2, 31, 31)).copy()
    A5 = _run(oracle, x, eps, 5, V=eye)
    assert np.abs(np.einsum("bhi,bhij->bh", x["mq"], A5) - 1.0).max() <= 1e-12
    A = _run(oracle, x, eps, 3000, V=eye)
    assert np.abs(A.sum(axis=-1) - 1.0).max() <= 1e-10
    assert np.abs(np.einsum("bhi,bhij->bhj", x["mq"], A) - x["mk"]).max() <= 1e-10


def test_zero_mass_tokens_are_padding(oracle):
    x, eps, iters = _case()
    base = _run(oracle, x, eps, iters)
    rng = np.random.default_rng(9)
    # three extra keys of mass zero, any content: the output does not change
    K2 = np.concatenate([x["K"], rng.standard_normal((2, 2, 3, 8))], axis=2)
    V2 = np.concatenate([x["V"], rng.standard_normal((2, 2, 3, 6))], axis=2)
    mk2 = np.concatenate([x["mk"], np.zeros((2, 2, 3))], axis=2)
    assert np.abs(_run(oracle, x, eps, iters, K=K2, V=V2, mk=mk2) - base).max() <= 1e-12
    # two extra queries of mass zero: the other rows do not change, and the new rows are still averages
    Q2 = np.concatenate([x["Q"], rng.standard_normal((2, 2, 2, 8))], axis=2)
    mq2 = np.concatenate([x["mq"], np.zeros((2, 2, 2))], axis=2)
    out = _run(oracle, x, eps, iters, Q=Q2, mq=mq2)
    assert np.abs(out[:, :, :20] - base).max() <= 1e-12
    ones = _run(oracle, x, eps, 3000, Q=Q2, mq=mq2, V=np.ones_like(x["V"]))     # converged: every row sums to one
    assert np.abs(ones - 1.0).max() <= 1e-10


def test_one_pivot_gives_the_weighted_mean_of_the_values(oracle):
    x, eps, iters = _case(r=1)
    out = _run(oracle, x, eps, iters)
    want = np.einsum("bhj,bhjc->bhc", x["mk"], x["V"])[:, :, None, :]
    assert np.abs(out - want).max() <= 1e-12
