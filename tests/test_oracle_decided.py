"""Pins of oracle.loss_grad_decided (the training step with relu decisions given by the caller, plus a
report of every pre-activation) and of the way the gradient tests use it (tests/relu_decisions.py)."""
import numpy as np
import pytest

import synth_inputs as si
from tests import dense_ref as dr
from tests import float32_yardstick as fy
from tests import relu_decisions as rd
from tests import train_cases as tc


def _small_case(seed=4, n=28, p=32, T=3, S=3):
    g = si.erdos_renyi_gnp(n, 0.2, seed)
    g.w = si.signed_edge_weights(g, seed, 1.0)
    theta = si.thetas(p, seed + 1, 0.2)
    x = si.node_flags(g.n, 0.3, seed + 2, n_states=S)
    action, target = si.training_batch(x, seed + 3)
    return g, theta, x, T, action, target


def _close(a, b, tol=1e-11):
    return np.max(np.abs(a - b)) <= tol * max(1.0, float(np.max(np.abs(b))))


def test_without_decisions_it_is_loss_grad(oracle_mod):
    g, theta, x, T, action, target = _small_case()
    l0, q0, g0 = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target)
    l1, q1, g1, pre = oracle_mod.loss_grad_decided(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target)
    assert l0 == l1 and np.array_equal(q0, q1)
    for k in si.THETA_NAMES:          # (the order of the OpenMP partial sums varies between calls)
        assert _close(g1[k], g0[k]), k
    # the reported pre-activations are those of Eq. 1: their positive part is the embedding of every round
    for b in range(x.shape[0]):
        _, hist = oracle_mod.embed(g.rowptr, g.colidx, g.w, theta, x[b], T, history=True)
        assert np.array_equal(np.maximum(pre["z"][b], 0.0), hist)
    # the summed magnitudes bound the pre-activations, and equal them where nothing cancels
    assert (np.abs(pre["z"]) <= pre["zs"] * (1 + 1e-12)).all() and (np.abs(pre["h"]) <= pre["hs"] * (1 + 1e-12)).all()
    # deciding every unit the way the definition does changes nothing
    force = (pre["z"] > 0).astype(np.int8)
    fh = (pre["h"] > 0).astype(np.int8)
    l2, q2, g2, _ = oracle_mod.loss_grad_decided(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target,
                                                 force=force, force_head=fh)
    assert l2 == l0
    for k in si.THETA_NAMES:
        assert _close(g2[k], g0[k]), k


def test_magnitudes_against_the_dense_form(oracle_mod):
    g, theta, x, T, action, target = _small_case(seed=9, n=16, p=32, T=2, S=1)
    _, _, _, pre = oracle_mod.loss_grad_decided(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target)
    th = {k: np.asarray(v, dtype=np.float64) for k, v in theta.items()}
    adj, wm = si.dense_adjacency(g), si.dense_weights(g)
    e = dr.edge_term(adj, wm, th["theta4"])
    mu1 = dr.embed_dense(adj, wm, theta, x[0], 1)
    a = adj @ mu1
    zs2 = np.abs(np.outer(x[0], th["theta1"])) + np.abs(a) @ np.abs(th["theta2"]).T + np.abs(e) @ np.abs(th["theta3"]).T
    np.testing.assert_allclose(pre["zs"][0, 1], zs2, rtol=1e-12)
    z2 = np.outer(x[0], th["theta1"]) + a @ th["theta2"].T + e @ th["theta3"].T
    np.testing.assert_allclose(pre["z"][0, 1], z2, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("seed", [4, 11])
def test_decided_units_against_torch_autograd(oracle_mod, seed):
    import torch

    g, theta, x, T, action, target = _small_case(seed=seed)
    S, n, p = x.shape[0], g.n, theta["theta1"].shape[0]
    rng = np.random.default_rng(seed)
    # a few percent of the units decided at random, on or off, whatever the sign of their pre-activation
    force = np.where(rng.random((S, T, n, p)) < 0.03, rng.integers(0, 2, (S, T, n, p)), -1).astype(np.int8)
    fh = np.where(rng.random((S, 2, p)) < 0.1, rng.integers(0, 2, (S, 2, p)), -1).astype(np.int8)
    loss, qp, grads, _ = oracle_mod.loss_grad_decided(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target,
                                                      force=force, force_head=fh)
    l0, _, g0 = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target)
    assert abs(loss - l0) > 1e-6 * abs(l0)          # the decisions do change the result
    adj = torch.tensor(si.dense_adjacency(g))
    wm = torch.tensor(si.dense_weights(g))
    th_t = {k: torch.tensor(np.asarray(v, dtype=np.float64), requires_grad=True) for k, v in theta.items()}
    lt = dr.loss_torch_decided(adj, wm, th_t, torch.tensor(x.astype(np.float64)), T, action,
                               torch.tensor(target.astype(np.float64)), force, fh)
    lt.backward()
    assert abs(float(lt.detach()) - loss) <= 1e-11 * max(1.0, abs(loss))
    for k in si.THETA_NAMES:
        assert _close(grads[k], th_t[k].grad.numpy(), 1e-10), k


@pytest.mark.parametrize("kind,seed", [("ba", 1145), ("ba", 9145), ("er", 1145)])
def test_float32_misses_are_units_float32_cannot_decide(oracle_mod, kind, seed):
    # Draws next to a relu switch (the first two are the ones on which a plain float32 evaluation on this
    # machine's CPU missed the oracle's gradient by 1.5e-4 and 6e-4): the float32 decisions differ from the
    # definition's only at units whose pre-activation is below float32 resolution, and on that branch the
    # float32 gradient meets the oracle's at the usual bar.
    p, T, S = 64, 4, 16
    g, x, action, target = tc.inputs(kind, S)
    theta = si.thetas(p, seed, tc.theta_scale(kind))
    _, _, og = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
    _, _, yg, on, on_head = fy.loss_grad_float32(g, theta, x, T, action, target, decisions=True)
    outs, info = rd.decided_reference(oracle_mod, g, theta, x, T, action, target, on, on_head)
    plain, decided = fy.worst_gradient_error(yg, og), fy.worst_gradient_error(yg, outs[0][2])
    print(f"{kind}/{seed}: float32 vs oracle {plain:.2e}; on its own branch {decided:.2e}; {info}", flush=True)
    assert decided <= 1e-4
