"""The state-by-state row order of the embedding rounds (chosen by size; forced here through
s2v_set_sliced_min_bytes) against the oracle and against the node-by-node order, for minibatch sizes that are
multiples of 16 (where it replaces the 16-state tiles) and for others (where it replaces the memory order)."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu
from tests import train_cases as tc

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.mark.parametrize("kind,p,T,S", [("er", 64, 4, 16), ("ba", 32, 3, 32), ("batch", 64, 5, 16), ("hub", 64, 4, 16),
                                        ("er", 64, 4, 3), ("ba", 32, 4, 8), ("hub", 64, 3, 24), ("batch", 32, 4, 17)])
def test_sliced_forward_matches_oracle(oracle_mod, kind, p, T, S):
    print(f"case sliced forward kind={kind} p={p} T={T} S={S}", flush=True)
    if kind == "hub":
        g = si.star_graph(700)             # one row far beyond the long-row threshold
        g.w = si.symmetric_edge_weights(g, 2, 0.5, 1.5)
    else:
        g = tc.graph(kind, 3)
    x = si.node_flags(g.n, 0.1, 4, n_states=S)
    theta = si.thetas(p, 11 + p + T, 0.05)
    dev = gu.Device(g, p, T, S=S)
    dev.ctx.s2v_set_sliced_min_bytes(0)
    out = dev.forward(theta, x, save=True)
    for s in range(S):
        mu, gsum, q = gu.oracle_forward(oracle_mod, g, theta, x[s], T)
        assert gu.rel_err(out["mu"][:, s, :], mu) <= TOL
        assert gu.rel_err(out["gsum"][s], gsum) <= TOL
        assert gu.rel_err(out["q"][s], q) <= TOL
    assert np.array_equal(out["saved"][T - 1], out["mu"])


@pytest.mark.parametrize("S", [16, 3])
def test_sliced_training_matches_oracle_and_single_call(oracle_mod, S):
    kind, p, T = "ba", 64, 4
    g, x, action, target = tc.inputs(kind, S)
    theta = si.thetas(p, tc.stored_seeds()[(kind, p, T, S)], tc.theta_scale(kind))
    dev = gu.Device(g, p, T, S=S, training=True)
    dev.ctx.s2v_set_sliced_min_bytes(0)
    prm = dev.params(theta)
    loss2, qp2, grads2 = dev.train_iter(prm, x, action, target)
    loss1, qp1, grads1, _ = dev.loss_grad(prm, x, action, target)
    oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
    assert abs(loss2 - oloss) <= TOL * abs(oloss) and gu.rel_err(qp2, oqp) <= TOL
    for name in si.THETA_NAMES:
        assert gu.rel_err(grads2[name], ograds[name], whole=True) <= TOL, name
        assert np.array_equal(grads1[name], grads2[name]), name
    assert loss1 == loss2 and np.array_equal(qp1, qp2)
