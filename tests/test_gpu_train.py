"""GPU parity of the training step (forward with saved activations, loss, backward, SGD)
against the float64 oracle.  Bar: loss, predicted Q and every gradient tensor within 1e-4
relative error (same floored metric as the forward tests)."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu
from tests import train_cases as tc

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _case(kind, seed):
    return tc.graph(kind, seed)


def _check_grads(got, want, tol=TOL):
    worst = {}
    for name in si.THETA_NAMES:
        worst[name] = gu.rel_err(got[name], want[name], whole=True)
    print("gradient rel errors:", {k: f"{v:.2e}" for k, v in worst.items()}, flush=True)
    for name, e in worst.items():
        assert e <= tol, name


@pytest.mark.parametrize("kind", tc.KINDS)
@pytest.mark.parametrize("p,T,S", tc.SHAPES)
def test_loss_and_gradients_match_oracle(oracle_mod, kind, p, T, S):
    print(f"case train kind={kind} p={p} T={T} S={S}", flush=True)
    g, x, action, target = tc.inputs(kind, S)
    # The parameter seed is the stored one: the first draw whose float64 gradient has no relu jump within
    # float32 rounding of it (gu.thetas_clear_of_kinks; tests/test_train_seeds.py re-derives entries).
    seed = tc.stored_seeds()[(kind, p, T, S)]
    theta = si.thetas(p, seed, tc.theta_scale(kind))
    print(f"theta seed {seed}", flush=True)
    dev = gu.Device(g, p, T, S=S, training=True)
    prm = dev.params(theta)
    loss, qp, grads = dev.train_iter(prm, x, action, target)
    oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
    assert gu.rel_err(qp, oqp) <= TOL
    assert abs(loss - oloss) <= TOL * abs(oloss)
    _check_grads(grads, ograds)


@pytest.mark.parametrize("kind", tc.KINDS)
@pytest.mark.parametrize("p,T,S,weighted", [(64, 4, 16, False), (32, 3, 16, False), (32, 5, 16, True), (64, 3, 16, True),
                                            (64, 4, 3, False), (32, 2, 16, False), (32, 3, 32, False)])
def test_single_call_equals_forward_then_backward(kind, p, T, S, weighted):
    # s2v_loss_grad promises the results of s2v_embed_fwd + s2v_embed_bwd bit for bit, whether it takes
    # its short cut (16 states, one graph, T >= 3: no round-1 rows, mask words instead of mu^T) or not.
    print(f"case single call kind={kind} p={p} T={T} S={S} weighted={weighted}", flush=True)
    g, x, action, target = tc.inputs(kind, S)
    if kind == "ba":
        action = action.copy()
        action[0] = int(np.argmax(np.diff(g.rowptr)))      # an action node with a long row
    theta = si.thetas(p, 5 + p + T, tc.theta_scale(kind))
    dev = gu.Device(g, p, T, S=S, training=True, weighted_sum=weighted)
    prm = dev.params(theta)
    loss2, qp2, grads2 = dev.train_iter(prm, x, action, target)
    gsum2 = dev.last_gsum
    loss1, qp1, grads1, gsum1 = dev.loss_grad(prm, x, action, target)
    assert loss1 == loss2 and np.array_equal(qp1, qp2) and np.array_equal(gsum1, gsum2)
    for name in si.THETA_NAMES:
        assert np.array_equal(grads1[name], grads2[name]), name


def test_sgd_iterations_follow_oracle(oracle_mod):
    # Sec. 4.5.2: several forward/backward/update iterations on the same minibatch.
    # Small parameters and the paper's learning rate (1e-5, Sec. 6.1) keep the four steps stable.
    p, T, S, iters, lr = 64, 3, 4, 4, 1e-5
    g = _case("er", 5)
    theta = si.thetas(p, 9, 0.03)
    x = si.node_flags(g.n, 0.1, 4, n_states=S)
    action, target = si.training_batch(x, 6)
    dev = gu.Device(g, p, T, S=S, training=True)
    prm = dev.params(theta)
    th = {k: v.astype(np.float64) for k, v in theta.items()}
    losses = []
    for it in range(iters):
        loss, _, grads = dev.train_iter(prm, x, action, target, lr=lr)
        oloss, _, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, x, T, action, target)
        th = oracle_mod.sgd(th, ograds, lr)
        print(f"iter {it}: loss gpu {loss:.6g} oracle {oloss:.6g}", flush=True)
        assert abs(loss - oloss) <= 5 * TOL * abs(oloss)
        losses.append(oloss)
    assert losses[-1] < losses[0]
    got = prm.to_numpy()
    for name in si.THETA_NAMES:
        assert gu.rel_err(got[name], th[name], whole=True) <= TOL, name


def test_sgd_step_is_exact_axpy():
    import torch

    import paper_2105_08764_amd as s2v

    p = 32
    theta = si.thetas(p, 1)
    grad = si.thetas(p, 2, 1.0)
    ctx = s2v.Context()
    prm, grd = s2v.Params.from_numpy(theta), s2v.Params.from_numpy(grad)
    ctx.s2v_sgd_step(prm, grd, 0.125)
    torch.cuda.synchronize()
    got = prm.to_numpy()
    for name in si.THETA_NAMES:
        want = theta[name].astype(np.float64) - 0.125 * grad[name].astype(np.float64)
        assert np.array_equal(got[name], want.astype(np.float32)), name   # lr is a power of two: exact in fp32


def test_training_config5_scaled(oracle_mod):
    # Four SGD iterations at the configuration's lr = 1e-3.  With theta ~ N(0, 0.1^2) the scores
    # are in the thousands while targets are N(0,1), so the loss and the parameters grow from
    # step to step (a property of the workload, not of the kernels).  Each iteration is therefore
    # compared on its own: the oracle starts from the parameters the GPU holds at that point.
    w = si.config(5, 0.01)
    g = w.graph
    print(f"config 5 scaled: n={g.n} nnz={g.nnz} S={w.x.shape[0]}", flush=True)
    dev = gu.Device(g, w.p, w.T, S=w.x.shape[0], training=True)
    prm = dev.params(w.theta)
    compared = 0
    for it in range(w.iters):
        th = {k: v.astype(np.float64) for k, v in prm.to_numpy().items()}
        oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, w.x, w.T, w.action, w.target)
        gmax = max(float(np.abs(v).max()) for v in ograds.values())
        print(f"iter {it}: oracle loss {oloss:.6g} max|grad| {gmax:.3g}", flush=True)
        if not np.isfinite(oloss) or oloss > 1e30 or gmax > 1e30:
            break                                   # beyond float32 range: nothing left to compare
        loss, qp, grads = dev.train_iter(prm, w.x, w.action, w.target, lr=w.lr)
        assert gu.rel_err(qp, oqp) <= TOL and abs(loss - oloss) <= TOL * abs(oloss)
        _check_grads(grads, ograds)
        want = oracle_mod.sgd(th, ograds, w.lr)
        got = prm.to_numpy()
        for name in si.THETA_NAMES:
            assert gu.rel_err(got[name], want[name], whole=True) <= TOL, name
        compared += 1
    assert compared >= 1


@pytest.mark.parametrize("S", [8, 24])
def test_row_mode_minibatch_on_a_scale_free_graph(oracle_mod, S):
    # Minibatch sizes that are not a multiple of 16 on configuration 5's kind of graph (long rows of several
    # segments among them): every round in row mode, the last reversed round from the neighbours' scalars.
    w = si.config(5, 0.03)
    g = w.graph
    x = si.node_flags(g.n, 0.05, 2005, n_states=S)
    action, target = si.training_batch(x, 5005)
    assert int(np.diff(g.rowptr).max()) > 1024
    print(f"row-mode minibatch: n={g.n} nnz={g.nnz} S={S} longest row {int(np.diff(g.rowptr).max())}", flush=True)
    dev = gu.Device(g, w.p, w.T, S=S, training=True)
    loss, qp, grads = dev.train_iter(dev.params(w.theta), x, action, target)
    oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, w.theta, x, w.T, action, target)
    assert gu.rel_err(qp, oqp) <= TOL and abs(loss - oloss) <= TOL * abs(oloss)
    _check_grads(grads, ograds)


def test_adam_steps_match_oracle(oracle_mod):
    import torch

    import paper_2105_08764_amd as s2v

    p = 64
    theta = si.thetas(p, 1)
    ctx = s2v.Context()
    prm = s2v.Params.from_numpy(theta)
    m, v = s2v.Params.zeros_like(prm), s2v.Params.zeros_like(prm)
    th = {k: a.astype(np.float64) for k, a in theta.items()}
    om = {k: np.zeros_like(a) for k, a in th.items()}
    ov = {k: np.zeros_like(a) for k, a in th.items()}
    for step in (1, 2, 3, 4):
        grad = si.thetas(p, 10 + step, 0.5)
        ctx.s2v_adam_step(prm, s2v.Params.from_numpy(grad), m, v, step, 1e-3)
        # the oracle takes the hyper-parameters as the float32 values the library receives
        th, om, ov = oracle_mod.adam(th, grad, om, ov, step, float(np.float32(1e-3)), float(np.float32(0.9)),
                                     float(np.float32(0.999)), float(np.float32(1e-8)))
    torch.cuda.synchronize()
    got, gm, gv = prm.to_numpy(), m.to_numpy(), v.to_numpy()
    for name in si.THETA_NAMES:
        assert gu.rel_err(got[name], th[name], whole=True) <= 1e-5, name
        assert gu.rel_err(gm[name], om[name], whole=True) <= 1e-5 and gu.rel_err(gv[name], ov[name], whole=True) <= 1e-5


def test_q_target_matches_oracle(oracle_mod):
    import torch

    parts = [si.barabasi_albert(n, 2, 3 + i) if n > 2 else si.edgeless(n) for i, n in enumerate((700, 1, 1500, 40))]
    g = si.block_diagonal(parts)
    S, p, T = 5, 32, 3
    theta = si.thetas(p, 2)
    x_next = si.node_flags(g.n, 0.3, 9, n_states=S)
    x_next[3, g.graph_off[3]:g.graph_off[4]] = 1.0            # one state whose graph has no candidate left
    action = np.array([5, 700, 900, g.graph_off[3] + 2, 100], dtype=np.int32)
    reward = np.random.default_rng(0).normal(size=S).astype(np.float32)
    dev = gu.Device(g, p, T, S=S)
    out = dev.forward(theta, x_next)
    tgt = torch.full((S,), float("nan"), device="cuda")
    dev.ctx.s2v_q_target(dev.graph, dev.last["q"], dev.last["x"], None, torch.from_numpy(action).cuda(),
                         torch.from_numpy(reward).cuda(), 0.9, S, tgt, dev.ws)
    torch.cuda.synchronize()
    # given the GPU's own float32 scores the maximum is exact; the sum is one float32 rounding away
    want = oracle_mod.q_target(g.graph_off, out["q"], x_next, None, action, reward, np.float32(0.9))
    np.testing.assert_allclose(tgt.cpu().numpy(), want, rtol=3e-7, atol=1e-30)
    assert tgt.cpu().numpy()[3] == reward[3]
    # and against the oracle's own float64 scores
    q64 = np.stack([gu.oracle_forward(oracle_mod, g, theta, x_next[s], T)[2] for s in range(S)])
    want64 = oracle_mod.q_target(g.graph_off, q64, x_next, None, action, reward, 0.9)
    assert gu.rel_err(tgt.cpu().numpy(), want64) <= 1e-4
