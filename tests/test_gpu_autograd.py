"""The torch.autograd glue (paper_2509_23436_amd.autograd) on the GPU: gradients that arrive through
loss.backward(), with ordinary torch operations before and after the library call, against the
float64 backward oracle driven through the same chain."""
import dataclasses

import numpy as np
import pytest

from paper_2509_23436_amd import synth
from util import rel_max_err

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS


@pytest.mark.parametrize("cls", [False, True])
def test_gradients_through_loss_backward_match_the_oracle(cls):
    import torch
    from oracle import lot_oracle_bwd
    from paper_2509_23436_amd import autograd
    w = dataclasses.replace(W["tiny"], B=2, H=3, n=150, d=32, r=8, iters=5, seed=90)
    x = synth.make_inputs(w)
    rng = np.random.default_rng(91)
    logits = rng.standard_normal(x["beta"].shape).astype(np.float32)      # beta = softmax(logits): a learnable mass
    mix = (rng.standard_normal((w.d, w.d)) / np.sqrt(w.d)).astype(np.float32)   # an output projection after the attention

    # float64 chain on the CPU: the oracle's forward inside ordinary torch operations
    t = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in
         dict(Q=x["Q"], K=x["K"], V=x["V"], Z=x["Z"], logits=logits).items()}
    beta64 = torch.softmax(t["logits"], dim=-1)
    if cls:
        bc = torch.full((w.B, w.H), 0.8, dtype=torch.float64)
        O64 = lot_oracle_bwd.forward_cls(t["Q"], t["K"], t["V"], t["Z"], beta64, w.eps, w.iters, bc)
    else:
        O64 = lot_oracle_bwd.forward(t["Q"], t["K"], t["V"], t["Z"], beta64, w.eps, w.iters)
    loss64 = ((O64 @ torch.tensor(mix, dtype=torch.float64)) ** 2).sum()
    ref = torch.autograd.grad(loss64, list(t.values()))

    d = {k: torch.tensor(np.asarray(v, dtype=np.float32), device="cuda", requires_grad=True) for k, v in
         dict(Q=x["Q"], K=x["K"], V=x["V"], Z=x["Z"], logits=logits).items()}
    beta = torch.softmax(d["logits"], dim=-1)
    if cls:
        O = autograd.lot_attention_cls(d["Q"], d["K"], d["V"], d["Z"], beta, w.eps, w.iters, 0.8)
    else:
        O = autograd.lot_attention(d["Q"], d["K"], d["V"], d["Z"], beta, w.eps, w.iters)
    loss = ((O @ torch.tensor(mix, device="cuda")) ** 2).sum()
    loss.backward()
    torch.cuda.synchronize()
    assert abs(float(loss.detach()) - float(loss64.detach())) <= 1e-4 * abs(float(loss64.detach()))
    for (name, leaf), r64 in zip(d.items(), ref):
        err = rel_max_err(leaf.grad.double().cpu().numpy(), r64.numpy())
        print("  d%-6s max-norm rel err %.3e" % (name, err), flush=True)
        assert err <= 1e-4, name


def test_cross_attention_gradients_through_loss_backward_match_the_oracle():
    import torch
    from oracle import lot_oracle_bwd
    from paper_2509_23436_amd import autograd
    B, H, n_q, n_k, d, r, eps, iters = 2, 2, 90, 140, 32, 8, 0.1, 5
    rng = np.random.default_rng(92)
    x = dict(Q=rng.standard_normal((B, H, n_q, d)) * d ** -0.5, K=rng.standard_normal((B, H, n_k, d)) * d ** -0.5,
             V=rng.standard_normal((B, H, n_k, d)), Z=rng.standard_normal((H, r, d)) * d ** -0.5,
             logits=rng.standard_normal((H, r)))
    x = {k: v.astype(np.float32) for k, v in x.items()}
    mass_q = rng.random((B, H, n_q)) + 0.1
    mass_k = rng.random((B, H, n_k)) + 0.1
    mass_k[:, :, n_k - 30:] = 0.0                                        # padding keys
    mass_q = (mass_q / mass_q.sum(-1, keepdims=True)).astype(np.float32)
    mass_k = (mass_k / mass_k.sum(-1, keepdims=True)).astype(np.float32)

    t = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in x.items()}
    O64 = lot_oracle_bwd.forward_cross(t["Q"], t["K"], t["V"], t["Z"], torch.softmax(t["logits"], dim=-1),
                                       torch.tensor(mass_q, dtype=torch.float64), torch.tensor(mass_k, dtype=torch.float64),
                                       eps, iters)
    loss64 = (O64 ** 2).sum()
    ref = torch.autograd.grad(loss64, list(t.values()))

    dv = {k: torch.tensor(v, device="cuda", requires_grad=True) for k, v in x.items()}
    O = autograd.lot_cross_attention(dv["Q"], dv["K"], dv["V"], dv["Z"], torch.softmax(dv["logits"], dim=-1), eps, iters,
                                     mass_q=torch.tensor(mass_q, device="cuda"), mass_k=torch.tensor(mass_k, device="cuda"))
    loss = (O ** 2).sum()
    loss.backward()
    torch.cuda.synchronize()
    assert abs(float(loss.detach()) - float(loss64.detach())) <= 1e-4 * abs(float(loss64.detach()))
    for (name, leaf), r64 in zip(dv.items(), ref):
        err = rel_max_err(leaf.grad.double().cpu().numpy(), r64.numpy())
        print("  d%-6s max-norm rel err %.3e" % (name, err), flush=True)
        assert err <= 1e-4, name


def test_workspaces_are_reused_and_a_failed_wait_is_raised_by_a_later_call(knobs):
    """One workspace per shape (a training step allocates none after its first iteration), and a wait
    between workgroups that gave up surfaces, without any device synchronisation by the glue, as an
    exception at a later call.  The wait is made to give up from the host (poll budget zero): every
    kernel still ends normally."""
    import torch
    from paper_2509_23436_amd import autograd, lot
    w = dataclasses.replace(W["long_4k"], B=1, H=2, iters=3, seed=93)       # several workgroups per problem
    x = synth.make_inputs(w)
    d = {k: torch.tensor(x[k], device="cuda").to(torch.bfloat16 if k in ("Q", "K", "V") else torch.float32)
         for k in ("Q", "K", "V", "Z", "beta")}
    for k in ("Q", "K", "V", "Z"):
        d[k].requires_grad_(True)
    autograd._workspaces.clear()
    for step in range(3):
        O = autograd.lot_attention(d["Q"], d["K"], d["V"], d["Z"], d["beta"], w.eps, w.iters)
        O.float().pow(2).sum().backward()
        if step == 0:
            held = {k: v.data_ptr() for k, v in autograd._workspaces.items()}
            assert len(held) == 2                                           # forward and backward
    assert {k: v.data_ptr() for k, v in autograd._workspaces.items()} == held
    autograd.check_pending(wait=True)                                       # nothing failed so far

    lot.lot_debug_set(lot.KNOB_SPIN_LIMIT, 0)
    with torch.no_grad():
        O = autograd.lot_attention(d["Q"], d["K"], d["V"], d["Z"], d["beta"], w.eps, w.iters)
    lot.lot_debug_set(lot.KNOB_SPIN_LIMIT, -1)
    with pytest.raises(RuntimeError, match="gave up"):
        autograd.check_pending(wait=True)
    assert torch.isnan(O.float()).any()
    # from now on the calls that leave the choice to the library run without any wait between workgroups
    # (one launch per pass): what made the wait fail cannot make them fail again
    assert autograd.stepwise_after_failure
    try:
        for k in ("Q", "K", "V", "Z"):
            d[k].grad = None
        O = autograd.lot_attention(d["Q"], d["K"], d["V"], d["Z"], d["beta"], w.eps, w.iters)
        O.float().pow(2).sum().backward()
        autograd.check_pending(wait=True)
        assert {key[-1] for key in autograd._workspaces} == {lot.PATH_AUTO, lot.PATH_STEPWISE}
        stepwise = [O.detach().float()] + [d[k].grad.float() for k in ("Q", "K", "V", "Z")]
        assert all(torch.isfinite(t).all() for t in stepwise)
    finally:
        autograd.stepwise_after_failure = False
    # ... and the persistent kernels on the same workspaces are unaffected by the earlier failure
    for k in ("Q", "K", "V", "Z"):
        d[k].grad = None
    O = autograd.lot_attention(d["Q"], d["K"], d["V"], d["Z"], d["beta"], w.eps, w.iters)
    O.float().pow(2).sum().backward()
    autograd.check_pending(wait=True)
    ordinary = [O.detach().float()] + [d[k].grad.float() for k in ("Q", "K", "V", "Z")]
    for a, b in zip(stepwise, ordinary):
        assert torch.isfinite(b).all()
        assert float((a - b).abs().max()) <= 2e-2 * float(b.abs().max())
