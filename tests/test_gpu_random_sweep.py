"""GPU parity on shapes nobody picked by hand: for each seed a variant (plain, [CLS], cross attention with
uniform, random or padded masses), a shape and the method's parameters are drawn from lists that mix tile
boundaries, ragged tails, few and many problems, and every regime of the dispatch rules; the forward output
and all gradients (of the path AUTO selects, and of FUSED and STEPWISE by name) are compared with the fp64 oracles, to the bars of the other parity tests
(fp32 I/O 1e-4, bf16 I/O 2e-2, max-norm relative).  The draws are seeded: the same cases on every run."""
import dataclasses
import sys

import numpy as np
import pytest

from paper_2509_23436_amd import synth
from util import to_device, to_host_f64

pytestmark = pytest.mark.gpu

SEEDS = list(range(36))


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _draw(seed, dtype, many_pivots=False):
    rng = np.random.default_rng(1000 * (1 if dtype == "f32" else 2) + seed + (500 if many_pivots else 0))
    case = {
        "kind": str(rng.choice(["plain", "cls", "cross", "cross"])),
        "d": int(rng.choice([32, 64])),
        "r": int(rng.choice([65, 96, 100, 128, 129, 200, 256]) if many_pivots else rng.choice([3, 7, 16, 31, 32, 33, 48, 64])),
        "B": int(rng.choice([1, 2, 3]) if many_pivots else rng.choice([1, 2, 3, 30, 90])),
        "H": int(rng.integers(1, 5)),
        "n": int(rng.choice([16, 17, 31, 32, 33, 64, 100, 197, 256, 257, 500, 513, 1000, 1500, 2049])),
        "iters": int(rng.choice([1, 2, 3, 5, 8, 10, 15, 16, 17, 20])),
        "eps": float(rng.choice([0.05, 0.1, 0.2])),
        "seed": int(rng.integers(0, 1 << 30)),
        "beta_cls": float(rng.choice([0.3, 1.0, 2.5])),
        "n_k": int(rng.choice([7, 40, 64, 300, 777, 2000])),
        "masses": str(rng.choice(["uniform", "random", "padded"])),
    }
    if case["B"] >= 30 and case["n"] > 520:
        case["n"] = 300            # (many problems: sizes the oracle still finishes in seconds)
    if case["B"] >= 30 and case["n_k"] > 520:
        case["n_k"] = 300
    return case


def _check(tag, got, ref, tol):
    g = to_host_f64(got)
    assert np.isfinite(g).all(), tag
    scale = np.abs(ref).max()
    err = np.abs(g - ref).max() / scale if scale > 1e-12 else np.abs(g).max()
    _say("  %-10s rel err %.3e (bar %.0e)" % (tag, err, tol))
    assert err <= tol, tag


@pytest.mark.parametrize("seed", SEEDS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_drawn_case_matches_the_oracles(dtype, seed):
    _run(_draw(seed, dtype), dtype, seed)


@pytest.mark.parametrize("seed", SEEDS[:16])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_drawn_case_with_more_than_64_pivots_matches_the_oracles(dtype, seed):
    """The same with 65 to 256 pivots: the kernels that take the pivots in groups of 64."""
    _run(_draw(seed, dtype, many_pivots=True), dtype, seed)


@pytest.mark.parametrize("seed", SEEDS[:12])
@pytest.mark.parametrize("path_name", ["fused", "stepwise"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_drawn_case_on_a_forced_path_matches_the_oracles(dtype, path_name, seed):
    """The tile kernels asked for by name: with waits between workgroups (FUSED) and with launch boundaries only
    (STEPWISE), whatever AUTO would have picked for the shape."""
    _run(_draw(seed, dtype, many_pivots=seed % 3 == 2), dtype, seed, path_name)


def _run(c, dtype, seed, path_name="auto"):
    import torch
    from oracle import lot_oracle, lot_oracle_bwd
    from paper_2509_23436_amd import lot
    path = {"auto": lot.PATH_AUTO, "fused": lot.PATH_FUSED, "stepwise": lot.PATH_STEPWISE}[path_name]
    bf16 = dtype == "bf16"
    tol = 2e-2 if bf16 else 1e-4
    _say("drawn case %s %d on path %s: %r" % (dtype, seed, path_name, c))
    w = dataclasses.replace(synth.WORKLOADS["tiny"], B=c["B"], H=c["H"], n=c["n"], d=c["d"], r=c["r"], eps=c["eps"],
                            iters=c["iters"], seed=c["seed"], dtype=dtype)
    x = synth.make_inputs(w)
    eps, iters = c["eps"], c["iters"]
    dO = np.random.default_rng(c["seed"] + 1).standard_normal(x["V"].shape).astype(np.float32)
    if bf16:
        dO = synth.round_to_bf16(dO)
    dev = to_device(dict(x, dO=dO), dtype)
    if c["kind"] == "plain":
        O_ref = lot_oracle.attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, threads=16)[0]
        refs, _ = lot_oracle_bwd.attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, dO)
        out = lot.lot_attention_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, path=path)
        got = lot.lot_attention_bwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, dev["dO"], path=path)
        names = ("dQ", "dK", "dV", "dZ", "dbeta")
    elif c["kind"] == "cls":
        bc = c["beta_cls"]
        O_ref = lot_oracle.attention_cls(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, bc, threads=16)
        refs, _ = lot_oracle_bwd.attention_cls_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], eps, iters, bc, dO)
        out = lot.lot_attention_cls_fwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, bc, path=path)
        got = lot.lot_attention_cls_bwd(dev["Q"], dev["K"], dev["V"], dev["Z"], dev["beta"], eps, iters, bc, dev["dO"], path=path)
        names = ("dQ", "dK", "dV", "dZ", "dbeta", "dbeta_cls")
    else:
        B, H, n, n_k, d = c["B"], c["H"], c["n"], c["n_k"], c["d"]
        r2 = np.random.default_rng(c["seed"] + 2)
        K = (r2.standard_normal((B, H, n_k, d)) * d ** -0.5).astype(np.float32)
        V = r2.standard_normal((B, H, n_k, d)).astype(np.float32)
        if bf16:
            K, V = synth.round_to_bf16(K), synth.round_to_bf16(V)
        if c["masses"] == "uniform":
            mq = mk = None
        else:
            mq, mk = r2.random((B, H, n)) + 0.1, r2.random((B, H, n_k)) + 0.1
            if c["masses"] == "padded":      # a padded tail on both sides: mass exactly zero
                mq[:, :, n - n // 4:] = 0.0
                mk[:, :, n_k - n_k // 3:] = 0.0
            mq = (mq / mq.sum(-1, keepdims=True)).astype(np.float32)
            mk = (mk / mk.sum(-1, keepdims=True)).astype(np.float32)
        mqo = mq if mq is not None else np.full((B, H, n), 1.0 / n)
        mko = mk if mk is not None else np.full((B, H, n_k), 1.0 / n_k)
        O_ref = lot_oracle.cross_attention(x["Q"], K, V, x["Z"], x["beta"], mqo, mko, eps, iters)
        refs, _ = lot_oracle_bwd.cross_attention_bwd(x["Q"], K, V, x["Z"], x["beta"], mqo, mko, eps, iters, dO)

        def on_device(a, io=False):
            if a is None:
                return None
            if io and bf16:
                return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(np.ascontiguousarray(a)).cuda()
        Kd, Vd = on_device(K, True), on_device(V, True)
        out = lot.lot_cross_attention_fwd(dev["Q"], Kd, Vd, dev["Z"], dev["beta"], eps, iters,
                                          mass_q=on_device(mq), mass_k=on_device(mk), path=path)
        got = lot.lot_cross_attention_bwd(dev["Q"], Kd, Vd, dev["Z"], dev["beta"], eps, iters, dev["dO"],
                                          mass_q=on_device(mq), mass_k=on_device(mk), path=path)
        names = ("dQ", "dK", "dV", "dZ", "dbeta")
    torch.cuda.synchronize()
    _check("O", out, O_ref, tol)
    for nm, g, ref in zip(names, got, refs):
        _check(nm, g, ref, tol)
