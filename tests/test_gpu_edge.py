"""GPU edge cases of the C interface: error codes (nothing is enqueued on an error), empty
inputs, run-to-run determinism.  Every kernel launched here exits normally."""
import ctypes

import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _status(exc):
    return exc.value.status


def test_error_codes():
    import torch

    import paper_2105_08764_amd as s2v

    g = si.erdos_renyi_gnp(200, 0.05, 1)
    dev = gu.Device(g, 32, 3, k_max=4)
    ctx, graph, ws = dev.ctx, dev.graph, dev.ws
    prm = dev.params(si.thetas(32, 1))
    x = torch.zeros((1, g.n), device="cuda")
    mu = torch.zeros((g.n, 1, 32), device="cuda")
    gsum = torch.zeros((1, 1, 32), device="cuda")
    q = torch.zeros((1, g.n), device="cuda")
    idx = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    val = torch.zeros((1, 4), device="cuda")
    cnt = torch.zeros((1,), dtype=torch.int32, device="cuda")

    # unsupported embedding size
    bad = s2v.Params(48, {k: torch.zeros(1, device="cuda") for k in s2v.THETA_NAMES})
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, bad, x, 3, 1, mu, None, gsum, ws)
    assert _status(e) == s2v.S2V_ERR_UNSUPPORTED
    # more than 2^31 - 1 rows (nodes times states): refused before anything is touched
    S_big = (1 << 31) // g.n + 1
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, prm, x, 3, S_big, mu, None, gsum, ws)
    assert _status(e) == s2v.S2V_ERR_UNSUPPORTED
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_policy_eval(graph, prm, x, 3, S_big, mu, gsum, q, ws)
    assert _status(e) == s2v.S2V_ERR_UNSUPPORTED
    # T < 1, S < 1
    for T, S in ((0, 1), (3, 0)):
        with pytest.raises(s2v.S2VError) as e:
            ctx.s2v_embed_fwd(graph, prm, x, T, S, mu, None, gsum, ws)
        assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # no output buffer at all
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, prm, x, 3, 1, None, None, gsum, ws)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # workspace too small
    small = ws[: 4096]
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, prm, x, 3, 1, mu, None, gsum, small)
    assert _status(e) in (s2v.S2V_ERR_WORKSPACE_TOO_SMALL, s2v.S2V_ERR_NOT_PREPARED)
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_graph_prepare(graph, small[:256])
    assert _status(e) == s2v.S2V_ERR_WORKSPACE_TOO_SMALL
    # a workspace that was never prepared
    other = torch.empty(dev.ws_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, prm, x, 3, 1, mu, None, gsum, other)
    assert _status(e) == s2v.S2V_ERR_NOT_PREPARED
    # misaligned workspace
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_embed_fwd(graph, prm, x, 3, 1, mu, None, gsum, ws[8:])
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # the one-call policy evaluation needs all three outputs and refuses what its two halves refuse
    for args in ((None, gsum, q), (mu, None, q), (mu, gsum, None)):
        with pytest.raises(s2v.S2VError) as e:
            ctx.s2v_policy_eval(graph, prm, x, 3, 1, args[0], args[1], args[2], ws)
        assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_policy_eval(graph, prm, x, 0, 1, mu, gsum, q, ws)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_policy_eval(graph, prm, x, 3, 1, mu, gsum, q, other)
    assert _status(e) == s2v.S2V_ERR_NOT_PREPARED
    # selection: k < 1; batch with k > 1
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_select_topk(graph, q[0], x[0], None, 0, idx, val, cnt, ws)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    gb = si.block_diagonal([si.edgeless(5), si.edgeless(7)])
    devb = gu.Device(gb, 32, 1, k_max=4)
    with pytest.raises(s2v.S2VError) as e:
        devb.ctx.s2v_select_topk(devb.graph, torch.zeros(12, device="cuda"), torch.zeros(12, device="cuda"), None, 2,
                                 torch.zeros((2, 2), dtype=torch.int32, device="cuda"),
                                 torch.zeros((2, 2), device="cuda"), torch.zeros(2, dtype=torch.int32, device="cuda"),
                                 devb.ws)
    assert _status(e) == s2v.S2V_ERR_UNSUPPORTED
    # gradient struct with another p
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_sgd_step(prm, s2v.Params.from_numpy(si.thetas(64, 1)), 0.1)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # bad graph offsets are caught by prepare (first offset must be 0, last must be N)
    off = torch.tensor([0, 3, 11], dtype=torch.int32, device="cuda")
    gbad = s2v.Graph(devb.graph.rowptr, devb.graph.colidx, None, off)
    with pytest.raises(s2v.S2VError) as e:
        devb.ctx.s2v_graph_prepare(gbad, devb.ws)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # after all those refusals the context still works
    ctx.s2v_embed_fwd(graph, prm, x, 3, 1, mu, None, gsum, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(mu).all()


def test_loss_grad_error_codes():
    import torch

    import paper_2105_08764_amd as s2v

    g = si.erdos_renyi_gnp(200, 0.05, 1)
    p, T, S = 32, 3, 16
    dev = gu.Device(g, p, T, S=S, training=True)
    ctx, graph, ws = dev.ctx, dev.graph, dev.ws
    prm = dev.params(si.thetas(p, 1))
    grads = s2v.Params.zeros_like(prm)
    x = torch.zeros((S, g.n), device="cuda")
    saved = torch.zeros((T, g.n, S, p), device="cuda")
    gsum = torch.zeros((S, 1, p), device="cuda")
    action = torch.zeros(S, dtype=torch.int32, device="cuda")
    target = torch.zeros(S, device="cuda")
    loss = torch.zeros(1, device="cuda")
    qp = torch.zeros(S, device="cuda")
    good = [saved, gsum, action, target, loss]
    for hole in range(5):
        a = list(good)
        a[hole] = None
        with pytest.raises(s2v.S2VError) as e:
            ctx.s2v_loss_grad(graph, prm, x, T, S, a[0], a[1], a[2], a[3], a[4], qp, grads, ws)
        assert _status(e) == s2v.S2V_ERR_INVALID_ARG, hole
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_loss_grad(graph, prm, x, 0, S, saved, gsum, action, target, loss, qp, grads, ws)
    assert _status(e) == s2v.S2V_ERR_INVALID_ARG
    # a workspace sized for inference only: refused before anything is launched, on the short-cut path
    # (16 states, T >= 3) as on the plain one
    small_bytes = ctx.s2v_workspace_bytes(graph, p, T, S, 1, False)
    assert small_bytes < dev.ws_bytes
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_loss_grad(graph, prm, x, T, S, saved, gsum, action, target, loss, qp, grads, ws[:small_bytes])
    assert _status(e) == s2v.S2V_ERR_WORKSPACE_TOO_SMALL
    other = torch.empty(dev.ws_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_loss_grad(graph, prm, x, T, S, saved, gsum, action, target, loss, qp, grads, other)
    assert _status(e) == s2v.S2V_ERR_NOT_PREPARED
    bad = s2v.Params(48, {k: torch.zeros(1, device="cuda") for k in s2v.THETA_NAMES})
    with pytest.raises(s2v.S2VError) as e:
        ctx.s2v_loss_grad(graph, bad, x, T, S, saved, gsum, action, target, loss, qp, grads, ws)
    assert _status(e) == s2v.S2V_ERR_UNSUPPORTED
    # q_pred is optional; and the context still works after the refusals
    ctx.s2v_loss_grad(graph, prm, x, T, S, saved, gsum, action, target, loss, None, grads, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(loss).all()


def test_empty_graph():
    import torch

    g = si.edgeless(0)
    dev = gu.Device(g, 32, 3, k_max=3)
    out = dev.forward(si.thetas(32, 1), np.zeros((1, 0), np.float32))
    assert out["mu"].shape == (0, 1, 32) and (out["gsum"] == 0).all()
    for k in (1, 3):
        idx, val, cnt = dev.select(np.zeros(0, np.float32), np.zeros(0, np.float32), None, k)
        assert cnt[0] == 0 and (idx == -1).all() and np.isneginf(val).all()
    gsum = torch.full((1, 1, 32), float("nan"), device="cuda")
    dev.ctx.s2v_policy_eval(dev.graph, dev.params(si.thetas(32, 1)), torch.zeros((1, 0), device="cuda"), 3, 1,
                            torch.zeros((0, 1, 32), device="cuda"), gsum, torch.zeros((1, 0), device="cuda"), dev.ws)
    torch.cuda.synchronize()
    assert (gsum == 0).all()


def test_single_node_and_single_round(oracle_mod):
    g = si.edgeless(1)
    theta = si.thetas(64, 2)
    for T in (1, 2):
        dev = gu.Device(g, 64, T)
        out = dev.forward(theta, np.ones((1, 1), np.float32))
        mu, gsum, q = gu.oracle_forward(oracle_mod, g, theta, np.ones(1), T)
        assert gu.rel_err(out["mu"][:, 0, :], mu) <= 1e-5 and gu.rel_err(out["q"][0], q) <= 1e-5


def test_results_are_deterministic():
    # fixed reduction trees and no float atomics: two runs give the same bits
    w = si.config(3, 0.02)
    g = w.graph
    S = 16
    x = si.node_flags(g.n, 0.05, 3, n_states=S)
    action, target = si.training_batch(x, 4)
    outs = []
    for _ in range(2):
        dev = gu.Device(g, w.p, w.T, S=S, k_max=50, training=True)
        loss, qp, grads = dev.train_iter(dev.params(w.theta), x, action, target)
        one = dev.loss_grad(dev.params(w.theta), x, action, target)      # the single call: the same bits again
        assert one[0] == loss and np.array_equal(one[1], qp)
        assert all(np.array_equal(one[2][k], grads[k]) for k in si.THETA_NAMES)
        dev1 = gu.Device(g, w.p, w.T, k_max=50)
        f = dev1.forward(w.theta, w.x)
        sel = dev1.select(f["q"][0], w.x[0], None, 50)
        outs.append((loss, qp, grads, f, sel))
    a, b = outs
    assert a[0] == b[0] and np.array_equal(a[1], b[1])
    for k in si.THETA_NAMES:
        assert np.array_equal(a[2][k], b[2][k]), k
    assert np.array_equal(a[3]["mu"], b[3]["mu"]) and np.array_equal(a[3]["q"], b[3]["q"])
    assert all(np.array_equal(u, v) for u, v in zip(a[4], b[4]))


def test_hub_rows_of_every_kind(oracle_mod):
    # a star of 3000 leaves plus a clique: rows of 3000 and of 299 entries cross the 256-entry hub
    # threshold in row mode (S = 3) and in node mode (S = 16), forward and backward
    star = si.star_graph(3000)
    clique = si.complete_graph(300)
    g = si.block_diagonal([star, clique])
    g.w = si.symmetric_edge_weights(g, 3, 0.5, 1.5)
    for S, p, T in ((3, 64, 3), (16, 32, 3), (16, 64, 4)):
        theta = si.thetas(p, 5, 0.01)
        x = si.node_flags(g.n, 0.3, 7, n_states=S)
        action, target = si.training_batch(x, 8)
        action[0] = 0                      # the hub itself is an action node
        action[1] = g.graph_off[1] + 5     # and a clique node
        x[0, 0] = 0
        dev = gu.Device(g, p, T, S=S, training=True)
        loss, qp, grads = dev.train_iter(dev.params(theta), x, action, target)
        oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
        assert gu.rel_err(qp, oqp) <= 1e-4 and abs(loss - oloss) <= 1e-4 * abs(oloss)
        for name in si.THETA_NAMES:
            assert gu.rel_err(grads[name], ograds[name], whole=True) <= 1e-4, (S, name)


@pytest.mark.parametrize("S,p,T", [(1, 64, 3), (1, 32, 2), (16, 64, 4), (16, 32, 3), (5, 32, 3)])
def test_row_lengths_around_the_long_row_and_segment_limits(oracle_mod, S, p, T):
    # One graph made of stars whose centres have 255, 256, 257 entries (the long-row threshold is 256),
    # 511, 512, 513 (one segment holds 512) and 1025 (three segments), plus a sparse part: forward through
    # the single-call policy evaluation and one training iteration, unit weights (flag-bit forms) and
    # signed weights (record forms).
    import torch

    print(f"case row lengths S={S} p={p} T={T}", flush=True)
    parts = [si.star_graph(n) for n in (255, 256, 257, 511, 512, 513, 1025)] + [si.erdos_renyi_gnp(90, 0.1, 4)]
    b = si.block_diagonal(parts)
    centres = b.graph_off[:-2]
    for signed in (False, True):
        g = si.Graph(b.n, b.rowptr, b.colidx, None, None)
        if signed:
            g.w = si.signed_edge_weights(g, 6, 1.0)
        assert sorted(np.diff(g.rowptr)[centres].tolist()) == [255, 256, 257, 511, 512, 513, 1025]
        theta = si.thetas(p, 31 + p + T, 0.01)
        x = si.node_flags(g.n, 0.2, 3, n_states=S)
        x[:, centres[2]] = 0
        action, target = si.training_batch(x, 9)
        action[0] = centres[2]                      # the 257-entry row is an action node
        dev = gu.Device(g, p, T, S=S, training=True)
        xd = torch.from_numpy(x).cuda()
        mu = torch.full((g.n, S, p), float("nan"), device="cuda")
        gsum = torch.full((S, 1, p), float("nan"), device="cuda")
        q = torch.full((S, g.n), float("nan"), device="cuda")
        dev.ctx.s2v_policy_eval(dev.graph, dev.params(theta), xd, T, S, mu, gsum, q, dev.ws)
        torch.cuda.synchronize()
        mu, gsum, q = mu.cpu().numpy(), gsum.cpu().numpy(), q.cpu().numpy()
        for s_ in range(S):
            omu, ogs, oq = gu.oracle_forward(oracle_mod, g, theta, x[s_], T)
            assert gu.rel_err(mu[:, s_, :], omu) <= 1e-4
            assert gu.rel_err(gsum[s_], ogs) <= 1e-4
            assert gu.rel_err(q[s_], oq, scale=gu.q_term_scale(theta, ogs[0], omu)) <= 1e-4
        loss, qp, grads, _ = dev.loss_grad(dev.params(theta), x, action, target)
        oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, theta, x, T, action, target)
        assert abs(loss - oloss) <= 1e-4 * abs(oloss)
        for name in si.THETA_NAMES:
            assert gu.rel_err(grads[name], ograds[name], whole=True) <= 1e-4, (signed, name)


@pytest.mark.parametrize("batched", [False, True])
def test_star_with_100000_leaves(oracle_mod, batched):
    # One row of 10^5 entries (196 segments of the long-row pre-pass) next to 10^5 rows of one entry, alone and
    # as one block of a block-diagonal batch: single-state policy evaluation and a 16-state training iteration
    # (node-mode rounds, mask-word and fused reversed rounds, the hub as one of the action nodes).
    import torch

    print(f"case star 1e5 batched={batched}", flush=True)
    star = si.star_graph(100_000)
    if batched:
        g = si.block_diagonal([si.barabasi_albert(300, 3, 5), star, si.edgeless(1), si.erdos_renyi_gnp(200, 0.05, 6)])
        hub = int(g.graph_off[1])
    else:
        g, hub = star, 0
    assert int(np.diff(g.rowptr).max()) == 100_000 and int(np.diff(g.rowptr)[hub]) == 100_000
    g.w = si.symmetric_edge_weights(g, 3, 0.5, 1.5)
    p, T = 64, 3
    theta = si.thetas(p, 17, 0.01)
    # one state: embedding, graph sums, scores of every node
    x = si.node_flags(g.n, 0.1, 4)
    x[0, hub] = 0
    dev = gu.Device(g, p, T)
    out = dev.forward(theta, x)
    omu, ogs, oq = gu.oracle_forward(oracle_mod, g, theta, x[0], T)
    errs = (gu.rel_err(out["mu"][:, 0, :], omu), gu.rel_err(out["gsum"][0], ogs), gu.rel_err(out["q"][0], oq))
    print("  single state, rel errors mu/gsum/q:", errs, flush=True)
    assert max(errs) <= 1e-4
    idx, val, cnt = dev.select(out["q"][0], x[0], None, 1)
    oi, ov, oc = oracle_mod.select(g.graph_off, out["q"][0], x[0], None, 1)
    assert np.array_equal(idx, oi) and np.array_equal(cnt, oc)
    del dev
    torch.cuda.empty_cache()
    # sixteen states: one training iteration, both entry points
    S = 16
    x = si.node_flags(g.n, 0.1, 8, n_states=S)
    x[:, hub] = 0
    action, target = si.training_batch(x, 9)
    action[0] = hub
    if batched:
        action[1] = 5                                # a state whose action lies in another graph of the batch
    dev = gu.Device(g, p, T, S=S, training=True)
    prm = dev.params(theta)
    loss, qp, grads = dev.train_iter(prm, x, action, target)
    loss1, qp1, grads1, _ = dev.loss_grad(prm, x, action, target)
    assert loss1 == loss and np.array_equal(qp1, qp)
    oloss, oqp, ograds = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
    errs = {k: gu.rel_err(grads[k], ograds[k], whole=True) for k in si.THETA_NAMES}
    print("  16 states, gradient rel errors:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    assert gu.rel_err(qp, oqp) <= 1e-4 and abs(loss - oloss) <= 1e-4 * abs(oloss)
    for k in si.THETA_NAMES:
        assert np.array_equal(grads1[k], grads[k]), k
        assert errs[k] <= 1e-4, k


@pytest.mark.parametrize("weighted", [False, True])
def test_single_state_round2_over_solution_densities_and_without_symmetry(oracle_mod, weighted):
    # One state, T >= 3, static graph without long rows or negative weights: round 2 works from flag bits and the
    # rows' totals.  With a sparse, a dense and an empty partial solution, and on a pattern that is NOT symmetric
    # (a promise of the interface that the forward pass does not need).
    n, p, T = 5000, 64, 4
    g = si.erdos_renyi_gnp(n, 30.0 / n, 17)
    if weighted:
        g.w = si.symmetric_edge_weights(g, 5, 0.5, 1.5)
    theta = si.thetas(p, 31)
    for frac in (0.05, 0.6, 0.0):
        x = si.node_flags(n, frac, 8)
        dev = gu.Device(g, p, T, weighted_sum=weighted)
        out = dev.forward(theta, x)
        mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, theta, x[0], T, weighted=weighted)
        gsum, q = oracle_mod.q_scores(g.graph_off, theta, mu)
        errs = (gu.rel_err(out["mu"][:, 0, :], mu), gu.rel_err(out["q"][0], q))
        print(f"  round 2 from flag bits, weighted={weighted}, x density {frac}: {errs}", flush=True)
        assert max(errs) <= 1e-4, errs
    if weighted:
        return
    # not symmetric: drop the entries (v, u) with v > u of every third row
    keep = np.ones(g.nnz, dtype=bool)
    rows = np.repeat(np.arange(n), np.diff(g.rowptr))
    keep[(rows % 3 == 0) & (rows > g.colidx)] = False
    rp = np.zeros(n + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows[keep], minlength=n), out=rp[1:])
    ga = si.Graph(n=n, rowptr=rp, colidx=g.colidx[keep].copy())
    x = si.node_flags(n, 0.05, 8)
    out = gu.Device(ga, p, T).forward(theta, x)
    mu, gsum, q = gu.oracle_forward(oracle_mod, ga, theta, x[0], T)
    errs = (gu.rel_err(out["mu"][:, 0, :], mu), gu.rel_err(out["q"][0], q))
    print(f"  pattern without symmetry: {errs}", flush=True)
    assert max(errs) <= 1e-4, errs
