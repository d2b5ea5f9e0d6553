"""GPU parity of lot_cross_attention_fwd (n_q != n_k, token masses, zero-mass padding) against the
oracle, element by element.  Bars as for the plain forward: fp32 1e-4, bf16 I/O 2e-2."""
import numpy as np
import pytest

from paper_2509_23436_amd import synth
from util import rel_max_err, to_host_f64

pytestmark = pytest.mark.gpu


def _inputs(B, H, n_q, n_k, d, d_v, r, seed, bf16, masses):
    rng = np.random.default_rng(seed)
    x = {"Q": rng.standard_normal((B, H, n_q, d)) * d ** -0.5, "K": rng.standard_normal((B, H, n_k, d)) * d ** -0.5,
         "V": rng.standard_normal((B, H, n_k, d_v)), "Z": rng.standard_normal((H, r, d)) * d ** -0.5}
    x = {k: v.astype(np.float32) for k, v in x.items()}
    if bf16:
        x = {k: synth.round_to_bf16(v) for k, v in x.items()}
    b = rng.random((H, r)) + 0.2
    x["beta"] = (b / b.sum(axis=-1, keepdims=True)).astype(np.float32)
    if masses == "uniform":
        x["mq"], x["mk"] = None, None
    else:
        mq = rng.random((B, H, n_q)) + 0.1
        mk = rng.random((B, H, n_k)) + 0.1
        if masses == "padded":                       # the tails of every sequence are padding
            mq[:, :, n_q - n_q // 4:] = 0.0
            mk[:, :, n_k - n_k // 3:] = 0.0
            mk[:, :, 0] = 0.0
        x["mq"] = (mq / mq.sum(axis=-1, keepdims=True)).astype(np.float32)
        x["mk"] = (mk / mk.sum(axis=-1, keepdims=True)).astype(np.float32)
    return x


CASES = {
    "tiny_uniform": dict(B=1, H=2, n_q=40, n_k=70, d=32, d_v=32, r=8, seed=500, bf16=False, masses="uniform", eps=0.1, iters=8),
    "tiny_masses": dict(B=2, H=2, n_q=50, n_k=33, d=32, d_v=32, r=8, seed=501, bf16=False, masses="random", eps=0.1, iters=8),
    "padded_f32": dict(B=2, H=3, n_q=197, n_k=300, d=64, d_v=64, r=16, seed=502, bf16=False, masses="padded", eps=0.1, iters=10),
    "bf16_cross": dict(B=1, H=2, n_q=700, n_k=2100, d=64, d_v=64, r=64, seed=503, bf16=True, masses="random", eps=0.05, iters=5),
    "bf16_padded_d32": dict(B=2, H=3, n_q=1000, n_k=600, d=32, d_v=32, r=32, seed=504, bf16=True, masses="padded", eps=0.1, iters=10),
    "long_keys_bf16": dict(B=2, H=4, n_q=1024, n_k=9000, d=64, d_v=64, r=64, seed=506, bf16=True, masses="padded", eps=0.05, iters=6),
    "long_queries_bf16": dict(B=2, H=4, n_q=9000, n_k=500, d=64, d_v=64, r=32, seed=507, bf16=True, masses="uniform", eps=0.05, iters=6),
    "other_dims": dict(B=1, H=2, n_q=60, n_k=90, d=16, d_v=24, r=80, seed=505, bf16=False, masses="random", eps=0.1, iters=4),
    # uniform masses, short sides of different lengths: the wavefront-per-side kernels with several wavefronts per
    # side, some of them without a tile on the shorter side
    "short_queries_long_keys_bf16": dict(B=2, H=2, n_q=100, n_k=400, d=64, d_v=64, r=32, seed=508, bf16=True, masses="uniform", eps=0.05, iters=7),
    "long_queries_few_keys_bf16": dict(B=1, H=3, n_q=900, n_k=70, d=64, d_v=64, r=24, seed=509, bf16=True, masses="uniform", eps=0.1, iters=6),
    "ragged_sides_f32": dict(B=2, H=1, n_q=77, n_k=230, d=32, d_v=32, r=48, seed=499, bf16=False, masses="uniform", eps=0.1, iters=9),
    # more than 64 pivots: the grouped tile kernels with per-side sizes and masses (the last group ragged)
    "grouped_f32_r100": dict(B=1, H=2, n_q=150, n_k=333, d=32, d_v=32, r=100, seed=520, bf16=False, masses="random", eps=0.1, iters=5),
    "grouped_padded_f32_r128": dict(B=2, H=2, n_q=400, n_k=197, d=64, d_v=64, r=128, seed=521, bf16=False, masses="padded", eps=0.1, iters=4),
    "grouped_bf16_r256": dict(B=1, H=2, n_q=700, n_k=2100, d=64, d_v=64, r=256, seed=522, bf16=True, masses="padded", eps=0.05, iters=5),
    "grouped_uniform_bf16_r130": dict(B=2, H=1, n_q=3000, n_k=500, d=32, d_v=32, r=130, seed=523, bf16=True, masses="uniform", eps=0.1, iters=6),
}


def _paths(c, backward=False):
    tiles = c["d"] == c["d_v"] and c["d"] in (32, 64)
    # one register tile up to 64 pivots, groups of 64 up to 256 (backward: as far as its tables fit local memory)
    limit = 256 if (not backward or c["bf16"] or c["d"] == 32) else 128
    fused = tiles and c["r"] <= limit
    return ["reference", "fused"] if fused else ["reference"]


@pytest.mark.parametrize("name,path_name", [(nm, pn) for nm in CASES for pn in _paths(CASES[nm])])
def test_cross_attention_matches_oracle(name, path_name):
    import torch
    from oracle import lot_oracle
    from paper_2509_23436_amd import lot
    path = {"reference": lot.PATH_REFERENCE, "fused": lot.PATH_FUSED}[path_name]
    c = dict(CASES[name])
    eps, iters = c.pop("eps"), c.pop("iters")
    x = _inputs(**c)
    print("case %s path %s: %r" % (name, path_name, CASES[name]), flush=True)
    B, H, n_q, n_k = c["B"], c["H"], c["n_q"], c["n_k"]
    mq = x["mq"] if x["mq"] is not None else np.full((B, H, n_q), 1.0 / n_q)
    mk = x["mk"] if x["mk"] is not None else np.full((B, H, n_k), 1.0 / n_k)
    ref = lot_oracle.cross_attention(x["Q"], x["K"], x["V"], x["Z"], x["beta"], mq, mk, eps, iters)

    def dev(a, io=False):
        if a is None:
            return None
        if io and c["bf16"]:
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    out = lot.lot_cross_attention_fwd(dev(x["Q"], True), dev(x["K"], True), dev(x["V"], True), dev(x["Z"]),
                                      dev(x["beta"]), eps, iters, mass_q=dev(x["mq"]), mass_k=dev(x["mk"]), path=path)
    torch.cuda.synchronize()
    O = to_host_f64(out)
    assert np.isfinite(O).all()
    tol = 2e-2 if c["bf16"] else 1e-4
    err = rel_max_err(O, ref)
    print("  max-norm rel err %.3e (bar %.0e)" % (err, tol), flush=True)
    assert err <= tol


# ---- backward

BWD_CASES = {
    "tiny_uniform": dict(B=1, H=2, n_q=40, n_k=70, d=32, d_v=32, r=8, seed=510, bf16=False, masses="uniform", eps=0.1, iters=6),
    "tiny_masses": dict(B=2, H=2, n_q=50, n_k=33, d=32, d_v=32, r=8, seed=511, bf16=False, masses="random", eps=0.1, iters=6),
    "padded_f32": dict(B=2, H=3, n_q=197, n_k=300, d=64, d_v=64, r=16, seed=512, bf16=False, masses="padded", eps=0.1, iters=8),
    "bf16_cross": dict(B=1, H=2, n_q=700, n_k=1300, d=64, d_v=64, r=64, seed=513, bf16=True, masses="random", eps=0.05, iters=5),
    "bf16_padded_d32": dict(B=2, H=3, n_q=600, n_k=400, d=32, d_v=32, r=32, seed=514, bf16=True, masses="padded", eps=0.1, iters=6),
    "other_dims": dict(B=1, H=2, n_q=60, n_k=90, d=16, d_v=24, r=80, seed=515, bf16=False, masses="random", eps=0.1, iters=4),
    "equal_uniform_bf16": dict(B=1, H=2, n_q=500, n_k=500, d=64, d_v=64, r=32, seed=516, bf16=True, masses="uniform", eps=0.05, iters=5),
    # several chunks per pair on both sides, a different number of tiles on each
    "long_keys_bf16": dict(B=2, H=4, n_q=1024, n_k=6000, d=64, d_v=64, r=64, seed=517, bf16=True, masses="padded", eps=0.05, iters=4),
    "long_queries_f32": dict(B=1, H=2, n_q=5000, n_k=300, d=32, d_v=32, r=16, seed=518, bf16=False, masses="random", eps=0.1, iters=4),
    # more than 64 pivots: the grouped tile kernels with per-side sizes and masses
    "grouped_f32_r100": dict(B=1, H=2, n_q=150, n_k=333, d=32, d_v=32, r=100, seed=530, bf16=False, masses="random", eps=0.1, iters=5),
    "grouped_padded_f32_r128": dict(B=2, H=2, n_q=400, n_k=197, d=64, d_v=64, r=128, seed=531, bf16=False, masses="padded", eps=0.1, iters=4),
    "grouped_bf16_r256": dict(B=1, H=2, n_q=700, n_k=2100, d=64, d_v=64, r=256, seed=532, bf16=True, masses="padded", eps=0.05, iters=5),
    "grouped_uniform_bf16_r130": dict(B=2, H=1, n_q=3000, n_k=500, d=32, d_v=32, r=130, seed=533, bf16=True, masses="uniform", eps=0.1, iters=6),
}


@pytest.mark.parametrize("name,path_name", [(nm, pn) for nm in BWD_CASES for pn in _paths(BWD_CASES[nm], backward=True)])
def test_cross_backward_matches_oracle(name, path_name):
    import torch
    from oracle import lot_oracle_bwd
    from paper_2509_23436_amd import lot
    path = {"reference": lot.PATH_REFERENCE, "fused": lot.PATH_FUSED}[path_name]
    c = dict(BWD_CASES[name])
    eps, iters = c.pop("eps"), c.pop("iters")
    x = _inputs(**c)
    print("case %s path %s: %r" % (name, path_name, BWD_CASES[name]), flush=True)
    B, H, n_q, n_k = c["B"], c["H"], c["n_q"], c["n_k"]
    dO = np.random.default_rng(c["seed"] + 17).standard_normal((B, H, n_q, c["d_v"])).astype(np.float32)
    if c["bf16"]:
        dO = synth.round_to_bf16(dO)
    mq = x["mq"] if x["mq"] is not None else np.full((B, H, n_q), 1.0 / n_q)
    mk = x["mk"] if x["mk"] is not None else np.full((B, H, n_k), 1.0 / n_k)
    refs, _ = lot_oracle_bwd.cross_attention_bwd(x["Q"], x["K"], x["V"], x["Z"], x["beta"], mq, mk, eps, iters, dO)

    def dev(a, io=False):
        if a is None:
            return None
        if io and c["bf16"]:
            return torch.from_numpy(synth.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    ws = None
    outs = []
    for fill in (0x00, 0xA5):                       # twice on one workspace with different contents
        got = lot.lot_cross_attention_bwd(dev(x["Q"], True), dev(x["K"], True), dev(x["V"], True), dev(x["Z"]),
                                          dev(x["beta"]), eps, iters, dev(dO, True), mass_q=dev(x["mq"]),
                                          mass_k=dev(x["mk"]), workspace=ws, path=path)
        torch.cuda.synchronize()
        outs.append(got)
        if ws is None:
            shape = lot.lot_xshape(B, H, n_q, n_k, c["d"], c["d_v"], c["r"], 1 if c["bf16"] else 0)
            need = lot.lot_cross_attention_bwd_workspace_bytes(shape, iters, path)
            ws = torch.full((need,), fill ^ 0xFF, dtype=torch.uint8, device="cuda")
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                           b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32))
    assert lot.lot_workspace_status(ws) == 0
    tol = 2e-2 if c["bf16"] else 1e-4
    for nm, g, ref in zip(("dQ", "dK", "dV", "dZ", "dbeta"), outs[0], refs):
        g = to_host_f64(g)
        assert np.isfinite(g).all(), nm
        err = rel_max_err(g, ref)
        print("  %-5s max-norm rel err %.3e (bar %.0e)" % (nm, err, tol), flush=True)
        assert err <= tol, nm
    if c["masses"] == "padded":                     # padding keys: exactly no gradient
        pad = mk == 0.0
        for g in (outs[0][1], outs[0][2]):
            assert float(to_host_f64(g)[pad].__abs__().max()) == 0.0


# A side of one or two tokens and a small eps: some pivot is so far from every token of that side that the
# column sum of its row-normalised kernel entries leaves the fp32 range (the tile kernels sum in the
# linear domain), while its mass still has to be carried by those tokens.  A randomised sweep found these;
# AUTO sends sides of fewer than 16 tokens to the plain kernels, which work in the log domain throughout.
FEW_TOKENS = {
    "one_query": dict(B=2, H=3, n_q=1, n_k=2000, d=32, r=16, iters=1, eps=0.02, seed=143895000),
    "two_queries": dict(B=1, H=2, n_q=2, n_k=300, d=32, r=64, iters=1, eps=0.02, seed=981827532),
    "one_key": dict(B=3, H=3, n_q=4096, n_k=1, d=32, r=31, iters=2, eps=0.02, seed=963506464),
    "one_key_many_problems": dict(B=40, H=1, n_q=257, n_k=1, d=32, r=5, iters=1, eps=0.02, seed=310134833),
    "fifteen_keys": dict(B=2, H=2, n_q=300, n_k=15, d=64, r=33, iters=4, eps=0.02, seed=7),
}


@pytest.mark.parametrize("name", list(FEW_TOKENS))
def test_a_side_of_very_few_tokens_meets_the_bar_on_the_kernels_auto_picks(name):
    import dataclasses
    import torch
    from oracle import lot_oracle
    from paper_2509_23436_amd import lot
    c = FEW_TOKENS[name]
    w = dataclasses.replace(synth.WORKLOADS["tiny"], B=c["B"], H=c["H"], n=c["n_q"], d=c["d"], r=c["r"], eps=c["eps"],
                            iters=c["iters"], seed=c["seed"], dtype="f32")
    x = synth.make_inputs(w)
    rng = np.random.default_rng(c["seed"] + 2)
    K = (rng.standard_normal((c["B"], c["H"], c["n_k"], c["d"])) * c["d"] ** -0.5).astype(np.float32)
    V = rng.standard_normal((c["B"], c["H"], c["n_k"], c["d"])).astype(np.float32)
    mq = np.full((c["B"], c["H"], c["n_q"]), 1.0 / c["n_q"])
    mk = np.full((c["B"], c["H"], c["n_k"]), 1.0 / c["n_k"])
    ref = lot_oracle.cross_attention(x["Q"], K, V, x["Z"], x["beta"], mq, mk, c["eps"], c["iters"])
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()      # noqa: E731
    out = lot.lot_cross_attention_fwd(dev(x["Q"]), dev(K), dev(V), dev(x["Z"]), dev(x["beta"]), c["eps"], c["iters"])
    torch.cuda.synchronize()
    err = rel_max_err(to_host_f64(out), ref)
    print("  %s: max-norm rel err %.3e (bar 1e-4)" % (name, err), flush=True)
    assert err <= 1e-4
