"""The single-launch step of Alg. 3 on small graphs (s2v_policy_select: embed, score and select in one kernel,
one workgroup per graph, the embedding held in LDS) against the float64 oracle, and against the general
path (s2v_policy_eval + s2v_select_topk), which it must match up to float32 rounding."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _graph(kind, seed):
    if kind == "er1000":
        return si.erdos_renyi_gnp(1000, 0.01, seed)                     # the largest graph p = 32 allows is 1024 nodes
    if kind == "er512":
        return si.erdos_renyi_gnp(512, 0.02, seed)                      # the largest p = 64 allows
    if kind == "dense":
        return si.erdos_renyi_gnp(257, 0.4, seed)                       # rows of ~100 entries: several index chunks
    if kind == "star":
        return si.star_graph(400)                                       # one row of 400 entries, 400 of one
    if kind == "batch":
        parts = [si.barabasi_albert(n, 3, seed + i) if n > 3 else si.edgeless(n)
                 for i, n in enumerate((500, 1, 77, 0, 300, 2, 64, 512))]
        return si.block_diagonal(parts)
    if kind == "tiny":
        return si.erdos_renyi_gnp(5, 0.8, seed)
    raise ValueError(kind)


def _run(dev, theta, x, cand, k, T):
    import torch

    g = dev.g_np
    N, G, p = g.n, g.n_graphs, dev.p
    prm = dev.params(theta)
    xd = torch.from_numpy(x).cuda()
    cd = None if cand is None else torch.from_numpy(cand).cuda()
    out = {}
    for name in ("small", "general"):
        mu = torch.full((N, 1, p), float("nan"), device="cuda")
        gsum = torch.full((1, G, p), float("nan"), device="cuda")
        q = torch.full((1, N), float("nan"), device="cuda")
        idx = torch.full((G, k), -7, dtype=torch.int32, device="cuda")
        val = torch.full((G, k), float("nan"), device="cuda")
        cnt = torch.full((G,), -7, dtype=torch.int32, device="cuda")
        if name == "small":
            dev.ctx.s2v_policy_select(dev.graph, prm, xd[0], cd, T, k, mu, gsum, q, idx, val, cnt, dev.ws)
        else:
            dev.ctx.s2v_policy_eval(dev.graph, prm, xd, T, 1, mu, gsum, q, dev.ws)
            dev.ctx.s2v_select_topk(dev.graph, q[0], xd[0], cd, k, idx, val, cnt, dev.ws)
        torch.cuda.synchronize()
        out[name] = tuple(t.cpu().numpy() for t in (mu, gsum, q, idx, val, cnt))
    return out


@pytest.mark.parametrize("kind,p", [("er1000", 32), ("er512", 64), ("dense", 64), ("dense", 32), ("star", 64),
                                    ("batch", 64), ("batch", 32), ("tiny", 32)])
@pytest.mark.parametrize("T", [1, 2, 4])
def test_single_launch_step_matches_oracle(oracle_mod, kind, p, T):
    print(f"case small kind={kind} p={p} T={T}", flush=True)
    g = _graph(kind, 5)
    if kind in ("er512", "batch"):
        g.w = si.symmetric_edge_weights(g, 11, 0.5, 1.5)
    if kind == "dense":
        g.w = si.signed_edge_weights(g, 12, 1.0)
    theta = si.thetas(p, 50 + p + T, 0.1 if kind not in ("star", "dense") else 0.02)
    x = si.node_flags(g.n, 0.2, 6)
    ks = (1,) if g.n_graphs > 1 else (1, 3, 8)
    dev = gu.Device(g, p, T, k_max=8)
    dev.ctx.s2v_set_single_launch(1)          # always: one graph of this size would take the chain of launches
    mu_o, gsum_o, q_o = gu.oracle_forward(oracle_mod, g, theta, x[0], T)
    rng = np.random.default_rng(3)
    for k in ks:
        for cand in (None, (rng.random(g.n) < 0.5).astype(np.uint8), np.zeros(g.n, dtype=np.uint8)):
            out = _run(dev, theta, x, cand, k, T)
            mu, gsum, q, idx, val, cnt = out["small"]
            errs = (gu.rel_err(mu[:, 0, :], mu_o), gu.rel_err(gsum[0], gsum_o), gu.rel_err(q[0], q_o))
            assert max(errs) <= TOL, errs
            # selection: the exact rule on the kernel's own float32 scores
            oi, ov, oc = oracle_mod.select(g.graph_off, q[0], x[0], cand, k)
            assert np.array_equal(idx, oi) and np.array_equal(cnt, oc)
            assert np.array_equal(val, ov.astype(np.float32))
            # the general path computes the same values up to float32 rounding (each is within TOL of the oracle)
            mu2, gsum2, q2 = out["general"][:3]
            assert gu.rel_err(mu, mu2) <= 2 * TOL and gu.rel_err(gsum, gsum2) <= 2 * TOL and gu.rel_err(q, q2) <= 2 * TOL
    print("  rel errors mu/gsum/q:", errs, flush=True)


def test_single_launch_on_a_shrinking_graph(oracle_mod):
    # the loop's mutable graph: rows shrink (row_end) and the edge sums in the workspace head follow
    import torch

    g = si.erdos_renyi_gnp(600, 0.03, 9)
    g.w = si.symmetric_edge_weights(g, 2, 0.5, 1.5)
    p, T = 32, 3
    theta = si.thetas(p, 8, 0.05)
    dev = gu.Device(g, p, T, k_max=8)
    dev.ctx.s2v_set_single_launch(1)
    mut = dev.graph.mutable_copy()
    dev.ctx.s2v_graph_prepare(mut, dev.ws)
    x = si.node_flags(g.n, 0.15, 4)[0]
    xd = torch.from_numpy(x).cuda()
    cand = torch.zeros(g.n, dtype=torch.uint8, device="cuda")
    stats = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    dev.ctx.s2v_residual_update(mut, xd, None, None, 0, cand, stats, dev.ws)
    mu = torch.empty((g.n, 1, p), device="cuda")
    gsum = torch.empty((1, 1, p), device="cuda")
    q = torch.empty((1, g.n), device="cuda")
    idx = torch.empty((1, 4), dtype=torch.int32, device="cuda")
    val = torch.empty((1, 4), device="cuda")
    cnt = torch.empty((1,), dtype=torch.int32, device="cuda")
    dev.ctx.s2v_policy_select(mut, dev.params(theta), xd, cand, T, 4, mu, gsum, q, idx, val, cnt, dev.ws)
    torch.cuda.synchronize()
    rp, ci, ww = oracle_mod.residual_graph(g.rowptr, g.colidx, g.w, x)
    mu_o = oracle_mod.embed(rp, ci, ww, theta, x, T)
    gs_o, q_o = oracle_mod.q_scores(None, theta, mu_o)
    assert gu.rel_err(mu.cpu().numpy()[:, 0, :], mu_o) <= TOL and gu.rel_err(q.cpu().numpy()[0], q_o) <= TOL
    oi, ov, oc = oracle_mod.select(None, q.cpu().numpy()[0], x, cand.cpu().numpy(), 4)
    assert np.array_equal(idx.cpu().numpy(), oi) and np.array_equal(cnt.cpu().numpy(), oc)


@pytest.mark.parametrize("n,deg,p", [(1025, 10, 32), (3000, 450, 64), (16384, 6, 64), (16385, 6, 64)])
@pytest.mark.parametrize("T", [2, 3])
def test_larger_graphs_take_the_general_path_bit_for_bit(n, deg, p, T):
    # 1025 nodes at p = 32 no longer fit a compute unit: the call is s2v_policy_eval followed by s2v_select_topk.
    # Up to 16384 nodes the library runs the tail of the evaluation and the first stage of the selection as one
    # launch (from 16385 on as separate ones); the caller must see the bits of the two calls either way.
    print(f"case tail n={n} deg={deg} p={p} T={T}", flush=True)
    g = si.erdos_renyi_gnp(n, deg / n, 2)
    g.w = si.symmetric_edge_weights(g, 4, 0.5, 1.5)
    theta = si.thetas(p, 3, 0.05 if deg > 100 else 0.1)
    x = si.node_flags(g.n, 0.2, 6)
    dev = gu.Device(g, p, T, k_max=8)
    rng = np.random.default_rng(8)
    few = np.zeros(g.n, dtype=np.uint8)
    few[[3, n - 1]] = 1                                                 # fewer candidates than k, none in most chunks
    for k in (1, 2, 8):
        for cand in (None, (rng.random(g.n) < 0.5).astype(np.uint8), few, np.zeros(g.n, dtype=np.uint8)):
            out = _run(dev, theta, x, cand, k, T)
            for a, b in zip(out["small"], out["general"]):
                assert np.array_equal(a, b, equal_nan=True)


def test_single_launch_is_chosen_where_it_pays():
    # automatic choice: a batch of 64 graphs takes the single launch, one graph of 1000 nodes the chain of
    # launches; "never" and "always" override.  The two forms differ in the last bits of mu, which tells them apart.
    import torch

    parts = [si.erdos_renyi_gnp(300, 0.03, 40 + i) for i in range(64)]
    theta = si.thetas(32, 9)
    for g, expect_single in ((si.block_diagonal(parts), True), (si.erdos_renyi_gnp(1000, 0.01, 3), False)):
        x = si.node_flags(g.n, 0.2, 6)
        dev = gu.Device(g, 32, 3, k_max=8)
        got = {}
        for mode in (2, 1, 0):                                           # never, always, automatic
            dev.ctx.s2v_set_single_launch(mode)
            got[mode] = _run(dev, theta, x, None, 1, 3)["small"]
        same_as_single = all(np.array_equal(a, b) for a, b in zip(got[0], got[1]))
        same_as_chain = all(np.array_equal(a, b) for a, b in zip(got[0], got[2]))
        assert not np.array_equal(got[1][0], got[2][0])                  # the two forms round differently
        assert same_as_single == expect_single and same_as_chain == (not expect_single)
        assert np.array_equal(got[1][3], got[2][3])                      # and select the same nodes here
