"""Seeded sweep over combinations the hand-picked parity cases do not all reach: embedding size, rounds,
states, graph shape, weight signs, the weighted-sum and per-state-residual flags, each drawn at random
(fixed seeds, tests/sweep_cases.py).  Forward through s2v_policy_eval against the oracle; training through
s2v_loss_grad against s2v_embed_fwd + s2v_embed_bwd (bit for bit) and against the oracle."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu
from tests import sweep_cases as sc

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.mark.parametrize("case", range(sc.N_CASES))
def test_sweep_forward(oracle_mod, case):
    import torch

    c = sc.draw(case)
    print(f"case sweep fwd {case}: {c['desc']}", flush=True)
    g, p, T, S = c["g"], c["p"], c["T"], c["S"]
    theta = si.thetas(p, c["seed"] + 7, c["scale"])
    dev = gu.Device(g, p, T, S=S, state_residual=c["residual"], weighted_sum=c["weighted_sum"])
    xd = torch.from_numpy(c["x"]).cuda()
    mu = torch.full((g.n, S, p), float("nan"), device="cuda")
    gsum = torch.full((S, g.n_graphs, p), float("nan"), device="cuda")
    q = torch.full((S, g.n), float("nan"), device="cuda")
    dev.ctx.s2v_policy_eval(dev.graph, dev.params(theta), xd, T, S, mu, gsum, q, dev.ws)
    torch.cuda.synchronize()
    ref = sc.oracle_forward(oracle_mod, c, theta)
    mu, gsum, q = mu.cpu().numpy(), gsum.cpu().numpy(), q.cpu().numpy()
    offs = g.offsets()
    worst = 0.0
    for b in range(S):
        worst = max(worst, gu.rel_err(mu[:, b, :], ref["mu"][:, b, :]), gu.rel_err(gsum[b], ref["gsum"][b]))
        for gi in range(g.n_graphs):
            lo, hi = offs[gi], offs[gi + 1]
            if hi > lo:
                scale = gu.q_term_scale(theta, ref["gsum"][b, gi], ref["mu"][lo:hi, b, :])
                worst = max(worst, gu.rel_err(q[b, lo:hi], ref["q"][b, lo:hi], scale=scale))
    print(f"  worst rel err {worst:.2e}", flush=True)
    assert worst <= TOL


@pytest.mark.parametrize("case", range(sc.N_CASES))
def test_sweep_training(oracle_mod, case):
    c = sc.draw(case)
    print(f"case sweep train {case}: {c['desc']}", flush=True)
    g, p, T, S = c["g"], c["p"], c["T"], c["S"]
    x, action, target = sc.training_inputs(c)
    # the stored seed: the first parameter draw without a relu switch within float32 rounding, found by the
    # oracle alone (gu.thetas_clear_of_kinks; tests/test_train_seeds.py re-derives entries)
    seed = sc.stored_seeds()[case]
    theta = si.thetas(p, seed, c["scale"])
    dev = gu.Device(g, p, T, S=S, training=True, state_residual=c["residual"], weighted_sum=c["weighted_sum"])
    prm = dev.params(theta)
    loss2, qp2, grads2 = dev.train_iter(prm, x, action, target)
    loss1, qp1, grads1, _ = dev.loss_grad(prm, x, action, target)
    assert loss1 == loss2 and np.array_equal(qp1, qp2)
    for name in si.THETA_NAMES:
        assert np.array_equal(grads1[name], grads2[name]), name
    oloss, oqp, ograds = sc.oracle_loss_grad(oracle_mod, c, theta, x, action, target)
    assert abs(loss2 - oloss) <= TOL * max(abs(oloss), 1e-30)
    # (Q is a signed sum of 2p terms that can cancel: its error is measured against their magnitude)
    scales = sc.q_pred_scales(oracle_mod, c, theta, x, action)
    assert np.all(np.abs(qp2 - oqp) <= TOL * np.maximum(np.abs(oqp), 1e-2 * scales))
    worst = {n: gu.rel_err(grads2[n], ograds[n], whole=True) for n in si.THETA_NAMES}
    print("  gradient rel errors:", {k: f"{v:.1e}" for k, v in worst.items()}, flush=True)
    for name, e in worst.items():
        assert e <= TOL, name
