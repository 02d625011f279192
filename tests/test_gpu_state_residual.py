"""GPU parity of the per-state residual graphs of a training minibatch (the sub-graphs that
Tuples2Graphs rebuilds in Alg. 4): every state of the batch is embedded, scored and
differentiated on the graph minus the edges of its own solution nodes, without building those
graphs.  The oracle side builds each state's graph explicitly and runs it as a batch of one."""
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
        g = si.relabel(si.star_graph(700), np.random.default_rng(5).permutation(701))   # one long row
    elif kind == "batch":
        g = si.block_diagonal([si.barabasi_albert(n, 2, seed + i) if n > 2 else si.edgeless(n)
                               for i, n in enumerate((40, 1, 77, 1300, 64))])
    else:
        raise ValueError(kind)
    return g


def _states(g, S, frac, seed):
    x = si.node_flags(g.n, frac, seed, n_states=S)
    action = np.zeros(S, dtype=np.int32)
    rng = np.random.default_rng(seed + 1)
    for b in range(S):                              # the action is a node outside the state's solution
        free = np.flatnonzero(x[b] == 0)
        action[b] = free[rng.integers(len(free))]
    target = rng.normal(size=S).astype(np.float32)
    return x, action, target


@pytest.mark.parametrize("kind", ["er", "ba", "hub", "batch"])
@pytest.mark.parametrize("p,T,S", [(32, 1, 3), (64, 2, 16), (32, 3, 5), (64, 4, 2), (32, 2, 1)])
def test_forward_on_per_state_residual_graphs(oracle_mod, kind, p, T, S):
    print(f"case state-residual fwd kind={kind} p={p} T={T} S={S}", flush=True)
    g = _graph(kind, 11)
    theta = si.thetas(p, 5 + p + T, 0.1 if kind != "ba" else 0.05)
    x, _, _ = _states(g, S, 0.3, 17)
    if kind == "hub":
        x[0, np.argmax(np.diff(g.rowptr))] = 1.0    # state 0 removes the hub itself
    dev = gu.Device(g, p, T, S=S, state_residual=True)
    out = dev.forward(theta, x)
    ref = gu.oracle_per_state_residual(oracle_mod, g, theta, x.astype(np.float64), T)
    for name in ("mu", "gsum"):
        e = gu.rel_err(out[name].reshape(ref[name].shape), ref[name])
        print(f"  {name}: {e:.2e}", flush=True)
        assert e <= TOL, name
    # Q per (state, graph): with so many isolated nodes the graph half of Eq. 2 dwarfs the node half
    # and Q is what is left of two large terms, so the floor follows the size of those terms.
    for b in range(S):
        for gi in range(g.n_graphs):
            lo, hi = (0, g.n) if g.graph_off is None else (g.graph_off[gi], g.graph_off[gi + 1])
            if hi == lo:
                continue
            sc = gu.q_term_scale(theta, ref["gsum"][b, gi], ref["mu"][lo:hi, b, :])
            e = gu.rel_err(out["q"][b, lo:hi], ref["q"][b, lo:hi], scale=sc)
            assert e <= TOL, ("q", b, gi, e)


@pytest.mark.parametrize("kind", ["er", "ba", "hub", "batch"])
@pytest.mark.parametrize("p,T,S", [(32, 1, 3), (64, 2, 16), (32, 3, 5), (64, 4, 2), (32, 4, 16), (64, 3, 16)])
def test_gradients_on_per_state_residual_graphs(oracle_mod, kind, p, T, S):
    print(f"case state-residual train kind={kind} p={p} T={T} S={S}", flush=True)
    g = _graph(kind, 12)
    theta = si.thetas(p, 31 + p + T, 0.1 if kind != "ba" else 0.05)
    x, action, target = _states(g, S, 0.3, 23)
    dev = gu.Device(g, p, T, S=S, training=True, state_residual=True)
    prm = dev.params(theta)
    loss, qp, grads = dev.train_iter(prm, x, action, target)
    _, (oloss, oqp, ograds) = gu.oracle_per_state_residual(oracle_mod, g, theta, x.astype(np.float64), T,
                                                          action, target.astype(np.float64))
    assert gu.rel_err(qp, oqp) <= TOL
    assert abs(loss - oloss) <= TOL * abs(oloss)
    for name in si.THETA_NAMES:
        e = gu.rel_err(grads[name], ograds[name], whole=True)
        print(f"  d{name}: {e:.2e}", flush=True)
        assert e <= TOL, name


def test_empty_solutions_give_the_plain_graph(oracle_mod):
    # With no solution node in any state the residual graphs are the graph itself: both modes agree exactly.
    g = _graph("ba", 3)
    p, T, S = 32, 3, 4
    theta = si.thetas(p, 2, 0.05)
    x = np.zeros((S, g.n), dtype=np.float32)
    a = gu.Device(g, p, T, S=S, state_residual=True).forward(theta, x)
    b = gu.Device(g, p, T, S=S).forward(theta, x)
    for name in ("mu", "gsum", "q"):
        assert np.array_equal(a[name], b[name]), name
