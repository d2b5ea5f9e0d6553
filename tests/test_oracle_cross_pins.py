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


# ---- backward (oracle.lot_oracle_bwd.cross_attention_bwd)

def _pad(x, n_pad_q=3, n_pad_k=4):
    """The same problem with the last tokens turned into padding (mass zero, masses renormalised)."""
    y = dict(x)
    mq = x["mq"].copy(); mk = x["mk"].copy()
    mq[..., -n_pad_q:] = 0.0; mk[..., -n_pad_k:] = 0.0
    y["mq"] = mq / mq.sum(axis=-1, keepdims=True)
    y["mk"] = mk / mk.sum(axis=-1, keepdims=True)
    return y


def _grads(x, eps, iters, dO):
    from oracle import lot_oracle_bwd
    return lot_oracle_bwd.cross_attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], x["mq"], x["mk"], eps, iters, dO)


def test_forward_of_the_cross_backward_oracle_equals_the_cross_oracle(oracle):
    for kw, pad in ((dict(), False), (dict(), True), (dict(n_q=9, n_k=40, r=3, iters=1), False), (dict(eps=0.05), True)):
        x, eps, iters = _case(**kw)
        if pad:
            x = _pad(x)
        dO = np.zeros(x["Q"].shape[:3] + (x["V"].shape[-1],))
        _, O_t = _grads(x, eps, iters, dO)
        O_c = _run(oracle, x, eps, iters)
        assert np.abs(O_t - O_c).max() <= 1e-12 * max(1.0, np.abs(O_c).max())


def test_cross_gradients_match_central_differences_of_the_cross_oracle(oracle):
    for pad in (False, True):
        x, eps, iters = _case(n_q=11, n_k=14, r=4, iters=4)
        if pad:
            x = _pad(x, 2, 3)
        rng = np.random.default_rng(8)
        dO = rng.standard_normal(x["Q"].shape[:3] + (x["V"].shape[-1],))
        grads, _ = _grads(x, eps, iters, dO)
        loss = lambda y: float((_run(oracle, y, eps, iters) * dO).sum())     # noqa: E731
        h = 1e-6
        for name, g in zip(("Q", "K", "V", "Z", "beta"), grads):
            assert np.isfinite(g).all(), name
            for _ in range(3):
                v = rng.standard_normal(x[name].shape)
                if name == "beta":
                    v *= 0.1 * x["beta"]
                fd = (loss(dict(x, **{name: x[name] + h * v})) - loss(dict(x, **{name: x[name] - h * v}))) / (2 * h)
                an = float((g * v).sum())
                assert abs(fd - an) <= 2e-6 * max(1.0, abs(an), abs(fd)), (name, pad, fd, an)


def test_uniform_masses_and_equal_lengths_give_the_plain_backward(oracle):
    from oracle import lot_oracle_bwd
    x, eps, iters = _case(n_q=17, n_k=17)
    x["mq"] = np.full_like(x["mq"], 1.0 / 17)
    x["mk"] = np.full_like(x["mk"], 1.0 / 17)
    dO = np.random.default_rng(2).standard_normal(x["V"].shape)
    got, _ = _grads(x, eps, iters, dO)
    ref, _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, dO)
    for g, r_ in zip(got, ref):
        assert np.abs(g - r_).max() <= 1e-11 * max(1.0, np.abs(r_).max())


def test_padding_keys_get_no_gradient_and_can_be_dropped(oracle):
    x, eps, iters = _case()
    x = _pad(x, n_pad_q=1, n_pad_k=4)
    x["mq"] = _case()[0]["mq"]                         # queries: all real
    dO = np.random.default_rng(3).standard_normal(x["Q"].shape[:3] + (x["V"].shape[-1],))
    (dQ, dK, dV, dZ, db), _ = _grads(x, eps, iters, dO)
    assert np.abs(dK[:, :, -4:]).max() == 0.0 and np.abs(dV[:, :, -4:]).max() == 0.0
    short = dict(x, K=x["K"][:, :, :-4], V=x["V"][:, :, :-4], mk=x["mk"][:, :, :-4])
    (dQ2, dK2, dV2, dZ2, db2), _ = _grads(short, eps, iters, dO)
    for a, b in ((dQ, dQ2), (dK[:, :, :-4], dK2), (dV[:, :, :-4], dV2), (dZ, dZ2), (db, db2)):
        assert np.abs(a - b).max() <= 1e-12 * max(1.0, np.abs(b).max())
