"""GPU parity of the weighted neighbour sum (the aggregation step of Alg. 1 read as a product with
the weighted adjacency matrix) against the oracle's weighted reading: forward, gradients, long
rows, the inference loop, and the combination with per-state residual graphs."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _graph(kind, seed):
    if kind == "er":
        g = si.erdos_renyi_gnp(300, 0.05, seed)
        g.w = si.signed_edge_weights(g, seed, 1.0)
    elif kind == "ba":
        g = si.barabasi_albert(1500, 4, seed)
        g.w = si.symmetric_edge_weights(g, seed, 0.5, 1.5)
    elif kind == "hub":
        g = si.block_diagonal([si.star_graph(3000), si.complete_graph(300)])
        g.w = si.symmetric_edge_weights(g, seed, 0.25, 1.75)
    else:
        raise ValueError(kind)
    return g


def _scale(kind):
    return {"er": 0.1, "ba": 0.05, "hub": 0.01}[kind]


@pytest.mark.parametrize("kind", ["er", "ba", "hub"])
@pytest.mark.parametrize("p,T,S", [(64, 4, 1), (32, 2, 3), (64, 3, 16), (32, 4, 32), (64, 1, 2)])
def test_weighted_forward(oracle_mod, kind, p, T, S):
    print(f"case weighted fwd kind={kind} p={p} T={T} S={S}", flush=True)
    g = _graph(kind, 4)
    theta = si.thetas(p, 13 + p + T, _scale(kind))
    x = si.node_flags(g.n, 0.2, 5, n_states=S)
    dev = gu.Device(g, p, T, S=S, weighted_sum=True)
    out = dev.forward(theta, x)
    worst = 0.0
    differs = T == 1
    for b in range(S):
        mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, theta, x[b], T, weighted=True)
        gs, q = oracle_mod.q_scores(g.graph_off, theta, mu)
        worst = max(worst, gu.rel_err(out["mu"][:, b, :], mu), gu.rel_err(out["gsum"][b], gs))
        offs = g.offsets()
        for gi in range(g.n_graphs):
            lo, hi = offs[gi], offs[gi + 1]
            sc = gu.q_term_scale(theta, gs[gi], mu[lo:hi])
            worst = max(worst, gu.rel_err(out["q"][b, lo:hi], q[lo:hi], scale=sc))
        if not differs:
            plain = oracle_mod.embed(g.rowptr, g.colidx, g.w, theta, x[b], T)
            differs = np.abs(plain - mu).max() > 1e-3 * np.abs(mu).max()
    print(f"  worst rel err {worst:.2e}", flush=True)
    assert worst <= TOL
    assert differs, "the weighted and the plain reading coincide on this input: the case tests nothing"


@pytest.mark.parametrize("kind", ["er", "ba", "hub"])
@pytest.mark.parametrize("p,T,S", [(64, 4, 3), (32, 2, 16), (64, 3, 16), (32, 3, 1), (64, 1, 2), (32, 4, 16)])
def test_weighted_gradients(oracle_mod, kind, p, T, S):
    print(f"case weighted train kind={kind} p={p} T={T} S={S}", flush=True)
    g = _graph(kind, 6)
    theta = si.thetas(p, 19 + p + T, _scale(kind))
    x = si.node_flags(g.n, 0.15, 9, n_states=S)
    action, target = si.training_batch(x, 10)
    if kind == "hub":
        action[0] = 0                       # the long row itself is an action node
        x[0, 0] = 0
    dev = gu.Device(g, p, T, S=S, training=True, weighted_sum=True)
    loss, qp, grads = dev.train_iter(dev.params(theta), x, action, target)
    oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target,
                                              weighted=True)
    assert gu.rel_err(qp, oqp) <= TOL
    assert abs(loss - oloss) <= TOL * abs(oloss)
    for name in si.THETA_NAMES:
        e = gu.rel_err(grads[name], ograds[name], whole=True)
        print(f"  d{name}: {e:.2e}", flush=True)
        assert e <= TOL, name


def test_unit_weights_reduce_to_the_plain_sum():
    g = si.barabasi_albert(800, 3, 2)
    p, T, S = 32, 3, 2
    theta = si.thetas(p, 3, 0.05)
    x = si.node_flags(g.n, 0.2, 1, n_states=S)
    a = gu.Device(g, p, T, S=S, weighted_sum=True).forward(theta, x)          # no weights stored: w = 1
    g.w = np.ones(g.colidx.shape[0], dtype=np.float32)
    b = gu.Device(g, p, T, S=S, weighted_sum=True).forward(theta, x)
    c = gu.Device(g, p, T, S=S).forward(theta, x)
    for name in ("mu", "gsum", "q"):
        assert np.array_equal(a[name], c[name]) and np.array_equal(b[name], c[name]), name


@pytest.mark.parametrize("p,T,S", [(32, 3, 4), (64, 2, 16)])
def test_weighted_sum_on_per_state_residual_graphs(oracle_mod, p, T, S):
    g = _graph("ba", 8)
    theta = si.thetas(p, 23, 0.05)
    x = si.node_flags(g.n, 0.3, 12, n_states=S)
    rng = np.random.default_rng(3)
    action = np.array([rng.choice(np.flatnonzero(x[b] == 0)) for b in range(S)], dtype=np.int32)
    target = rng.normal(size=S).astype(np.float32)
    dev = gu.Device(g, p, T, S=S, training=True, state_residual=True, weighted_sum=True)
    loss, qp, grads = dev.train_iter(dev.params(theta), x, action, target)
    _, (oloss, oqp, ograds) = gu.oracle_per_state_residual(oracle_mod, g, theta, x.astype(np.float64), T, action,
                                                          target.astype(np.float64), weighted=True)
    assert gu.rel_err(qp, oqp) <= TOL and abs(loss - oloss) <= TOL * abs(oloss)
    for name in si.THETA_NAMES:
        assert gu.rel_err(grads[name], ograds[name], whole=True) <= TOL, name


def test_weighted_inference_loop_follows_the_oracle(oracle_mod):
    # Alg. 3 with the weighted sum: every policy evaluation of the native loop's solution path is
    # re-checked against the oracle from the same state, and the result is a vertex cover.
    import torch

    import paper_2105_08764_amd as s2v

    g = si.erdos_renyi_gnp(200, 0.05, 5)
    g.w = si.symmetric_edge_weights(g, 5, 0.5, 1.5)
    p, T = 32, 3
    theta = si.thetas(p, 9, 0.05)
    ctx = s2v.Context()
    graph = s2v.Graph(torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda(),
                      torch.from_numpy(g.w).cuda(), None, weighted_sum=True).mutable_copy()
    assert graph.weighted_sum
    ws = torch.empty(max(256, ctx.s2v_workspace_bytes(graph, p, T, 1, 8)), dtype=torch.uint8, device="cuda")
    ctx.s2v_graph_prepare(graph, ws)
    prm = s2v.Params.from_numpy(theta)
    N = g.n
    x = torch.zeros(N, device="cuda")
    mu = torch.empty((N, 1, p), device="cuda")
    gsum = torch.empty((1, 1, p), device="cuda")
    q = torch.empty((1, N), device="cuda")
    cand = torch.zeros(N, dtype=torch.uint8, device="cuda")
    sel_idx = torch.full((1, 8), -1, dtype=torch.int32, device="cuda")
    sel_val = torch.empty((1, 8), device="cuda")
    sel_cnt = torch.zeros(1, dtype=torch.int32, device="cuda")
    stats = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    x_ref = np.zeros(N)
    for step in range(N):
        n_steps, _, live = ctx.s2v_mvc_inference(graph, prm, x, T, False, 1, mu, gsum, q, cand, sel_idx, sel_val,
                                                 sel_cnt, stats, ws)
        if n_steps == 0:
            break
        rp, ci, ww = oracle_mod.residual_graph(g.rowptr, g.colidx, g.w, x_ref)
        omu = oracle_mod.embed(rp, ci, ww, theta, x_ref, T, weighted=True)
        _, oq = oracle_mod.q_scores(None, theta, omu)
        assert gu.rel_err(q.cpu().numpy()[0], oq, scale=gu.q_term_scale(theta, omu.sum(0), omu)) <= TOL
        x_ref = x.cpu().numpy().astype(np.float64)
        if live == 0:
            break
    rows = np.repeat(np.arange(N), np.diff(g.rowptr))
    assert ((x_ref[rows] != 0) | (x_ref[g.colidx] != 0)).all()
