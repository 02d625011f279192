"""Pins of the oracle's inference loop (Alg. 3 + the top-d selection of Sec. 4.5.1), no GPU."""
import os

import numpy as np
import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_adaptive_d_matches_the_papers_table(oracle_mod):
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "adaptive_d_table.txt"))
            if l.strip() and not l.startswith("#")]
    for c, n, d in rows:
        assert oracle_mod.adaptive_d(int(c), int(n)) == int(d), (c, n, d)


def test_residual_graph_against_dense_mask(oracle_mod):
    g = si.barabasi_albert(60, 3, 2)
    g.w = si.symmetric_edge_weights(g, 1, 0.5, 1.5)
    x = (np.random.default_rng(3).random(g.n) < 0.3).astype(np.float64)
    rp, ci, ww = oracle_mod.residual_graph(g.rowptr, g.colidx, g.w, x)
    alive = np.outer(x == 0, x == 0)
    want = si.dense_weights(g) * alive
    got = si.dense_weights(si.Graph(n=g.n, rowptr=rp, colidx=ci, w=ww))
    np.testing.assert_array_equal(got, want)


@pytest.mark.parametrize("adaptive", [False, True])
@pytest.mark.parametrize("kind", ["er", "ba", "batch"])
def test_loop_ends_in_a_vertex_cover(oracle_mod, kind, adaptive):
    if kind == "er":
        g = si.erdos_renyi_gnp(80, 0.08, 4)
    elif kind == "ba":
        g = si.barabasi_albert(120, 2, 5)
    else:
        g = si.block_diagonal([si.erdos_renyi_gnp(30, 0.2, 6), si.barabasi_albert(40, 2, 7), si.edgeless(3)])
    theta = si.thetas(8, 11, 0.3)
    x0 = np.zeros(g.n)
    x, steps, trace = oracle_mod.mvc_inference(g.rowptr, g.colidx, g.w, g.graph_off, theta, x0, 3, adaptive, 10_000)
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    assert ((x[rows] != 0) | (x[g.colidx] != 0)).all()            # every edge has an endpoint in the solution
    assert steps == len(trace) and steps >= 1
    lives = [t[3] for t in trace]
    assert all(a > b for a, b in zip(lives, lives[1:]))            # edges strictly decrease
    picked = np.concatenate([t[1] for t in trace])
    assert len(set(picked.tolist())) == len(picked) == int(x.sum())   # nobody is selected twice
    for d, chosen, n_cand, _ in trace:
        if g.n_graphs == 1:
            assert d == (oracle_mod.adaptive_d(n_cand, g.n) if adaptive else 1)
            assert len(chosen) == min(d, n_cand)
        else:
            assert d == 1 and 1 <= len(chosen) <= g.n_graphs


def test_loop_respects_a_partial_solution_and_max_steps(oracle_mod):
    g = si.star_graph(20)
    theta = si.thetas(8, 1, 0.3)
    x0 = np.zeros(g.n)
    x0[0] = 1.0                                                   # the hub already covers every edge
    x, steps, trace = oracle_mod.mvc_inference(g.rowptr, g.colidx, None, None, theta, x0, 2, False, 100)
    assert steps == 0 and np.array_equal(x, x0)
    g2 = si.cycle_graph(12)
    x, steps, _ = oracle_mod.mvc_inference(g2.rowptr, g2.colidx, None, None, theta, np.zeros(12), 2, False, 2)
    assert steps == 2 and x.sum() == 2
