"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test names the passage it leans on.  The paper prints no worked numerical
example (its figures are elided), so the pins are closed forms, recurrences on
vertex-transitive and two-orbit graphs, a dense-matrix brute force, explicit matrix
powers in the clip-free regime, invariances, a library sort, torch autograd on the
dense form and central finite differences.
"""
import numpy as np
import pytest

import synth_inputs as si
from tests import dense_ref as dr


def rand_theta(p, seed, std=0.3, positive=False):
    th = si.thetas(p, seed, std)
    if positive:
        th = {k: np.abs(v) for k, v in th.items()}
    return th


def relu(a):
    return np.maximum(a, 0.0)


# ---- P13: shapes -----------------------------------------------------------------

def test_parameter_count_matches_paper():
    # Sec. 5.1 item (3): the model has 4K^2 + 4K parameters.
    for p in (4, 32, 64):
        total = sum(int(np.prod(s)) for s in si.theta_shapes(p).values())
        assert total == 4 * p * p + 4 * p


# ---- P1: edgeless graph ----------------------------------------------------------

def test_edgeless_closed_form(oracle_mod):
    # Eq. (1) with N(v) empty: every round gives relu(theta1 * x_v); Alg. 1 starts from zero.
    p, n = 8, 17
    th = rand_theta(p, 1)
    g = si.edgeless(n)
    x = np.random.default_rng(0).normal(size=n)
    for T in (1, 2, 5):
        mu = oracle_mod.embed(g.rowptr, g.colidx, None, th, x, T)
        want = relu(np.outer(x, th["theta1"].astype(np.float64)))
        np.testing.assert_allclose(mu, want, rtol=0, atol=1e-15)
    # Eq. (2) closed form on top of it
    gsum, q = oracle_mod.q_scores(None, th, mu)
    t5, t6, t7 = (th[k].astype(np.float64) for k in ("theta5", "theta6", "theta7"))
    want_q = t5[:p] @ relu(t6 @ want.sum(0)) + relu(want @ t7.T) @ t5[p:]
    np.testing.assert_allclose(gsum[0], want.sum(0), rtol=1e-14)
    np.testing.assert_allclose(q, want_q, rtol=1e-13)


# ---- P2: one round has no neighbour-embedding term ---------------------------------

def test_single_round_closed_form(oracle_mod):
    p = 6
    th = rand_theta(p, 2)
    g = si.erdos_renyi_gnp(30, 0.2, 5)
    g.w = si.signed_edge_weights(g, 3, 2.0)
    x = np.random.default_rng(1).normal(size=g.n)
    mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, 1)
    t1, t3, t4 = (th[k].astype(np.float64) for k in ("theta1", "theta3", "theta4"))
    for v in range(g.n):
        ws = g.w[g.rowptr[v]:g.rowptr[v + 1]].astype(np.float64)
        e = relu(np.outer(ws, t4)).sum(0)
        np.testing.assert_allclose(mu[v], relu(t1 * x[v] + t3 @ e), rtol=1e-13, atol=1e-15)


# ---- P3: vertex-transitive graphs, uniform x and w: a p-dimensional recurrence ---------

@pytest.mark.parametrize("maker,deg", [(lambda: si.cycle_graph(11), 2), (lambda: si.complete_graph(9), 8)])
def test_regular_graph_recurrence(oracle_mod, maker, deg):
    p, T = 5, 4
    th = rand_theta(p, 3)
    g = maker()
    wval, xval = 0.7, 1.0
    mu, hist = oracle_mod.embed(g.rowptr, g.colidx, np.full(g.nnz, wval), th, np.full(g.n, xval), T, history=True)
    t1, t2, t3, t4 = (th[k].astype(np.float64) for k in ("theta1", "theta2", "theta3", "theta4"))
    c = t1 * xval + t3 @ (deg * relu(t4 * wval))
    m = np.zeros(p)
    for t in range(T):
        m = relu(c + deg * (t2 @ m))
        # automorphic nodes carry identical embeddings
        np.testing.assert_allclose(hist[t], np.tile(m, (g.n, 1)), rtol=1e-13, atol=1e-15)
    _, q = oracle_mod.q_scores(None, th, mu)
    assert np.ptp(q) <= 1e-12 * max(1.0, abs(q[0]))


# ---- P4: two-orbit graphs (star, complete bipartite): a 2-vector recurrence ------------

@pytest.mark.parametrize("a,b", [(1, 40), (3, 7), (1, 3000)])
def test_two_orbit_recurrence(oracle_mod, a, b):
    p, T = 4, 4
    th = rand_theta(p, 4, std=0.05 if b > 100 else 0.3)
    g = si.complete_bipartite(a, b)  # a == 1 is the star
    x = np.concatenate([np.full(a, 1.0), np.full(b, 0.0)])
    mu = oracle_mod.embed(g.rowptr, g.colidx, None, th, x, T)
    t1, t2, t3, t4 = (th[k].astype(np.float64) for k in ("theta1", "theta2", "theta3", "theta4"))
    e1 = relu(t4)
    ml, mr = np.zeros(p), np.zeros(p)
    for _ in range(T):
        ml, mr = relu(t1 * 1.0 + b * (t2 @ mr) + t3 @ (b * e1)), relu(a * (t2 @ ml) + t3 @ (a * e1))
    np.testing.assert_allclose(mu[:a], np.tile(ml, (a, 1)), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(mu[a:], np.tile(mr, (b, 1)), rtol=1e-12, atol=1e-14)


# ---- P5: dense adjacency brute force, 8..64 nodes --------------------------------------

@pytest.mark.parametrize("n,prob,seed", [(8, 0.5, 1), (23, 0.3, 2), (64, 0.1, 3), (64, 0.6, 4)])
def test_dense_brute_force_forward_and_q(oracle_mod, n, prob, seed):
    p, T = 7, 4
    th = rand_theta(p, 10 + seed)
    g = si.erdos_renyi_gnp(n, prob, seed)
    g.w = si.signed_edge_weights(g, seed, 1.5)
    x = np.random.default_rng(seed).normal(size=n)
    adj, wm = si.dense_adjacency(g), si.dense_weights(g)
    assert np.array_equal(adj, adj.T)
    mu, hist = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, T, history=True)
    want, want_hist = dr.embed_dense(adj, wm, th, x, T, history=True)
    for t in range(T):
        np.testing.assert_allclose(hist[t], want_hist[t], rtol=1e-11, atol=1e-13)
    assert (mu > 0).any() and (mu == 0).any()  # both branches of the relu are exercised
    _, q = oracle_mod.q_scores(None, th, mu)
    np.testing.assert_allclose(q, dr.q_dense(th, want), rtol=1e-11, atol=1e-13)


# ---- P6: clip-free regime: mu^T = sum_{j<T} A^j C (theta2^T)^j --------------------------

def test_linear_regime_matrix_powers(oracle_mod):
    p, T, n = 5, 4, 20
    th = rand_theta(p, 20, std=0.2, positive=True)
    g = si.erdos_renyi_gnp(n, 0.3, 7)
    g.w = np.abs(si.signed_edge_weights(g, 1, 1.0))
    x = np.abs(np.random.default_rng(3).normal(size=n))
    adj, wm = si.dense_adjacency(g), si.dense_weights(g)
    t1, t2, t3, t4 = (th[k].astype(np.float64) for k in ("theta1", "theta2", "theta3", "theta4"))
    C = np.outer(x, t1) + (wm.sum(1)[:, None] * t4[None, :]) @ t3.T  # all terms >= 0: no clipping anywhere
    want = sum(np.linalg.matrix_power(adj, j) @ C @ np.linalg.matrix_power(t2.T, j) for j in range(T))
    mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, T)
    np.testing.assert_allclose(mu, want, rtol=1e-12)


# ---- P9: Eq. (1)'s per-edge relu vs Alg. 1's relu of the summed product -----------------

def test_edge_term_forms(oracle_mod):
    p, n = 6, 25
    th = rand_theta(p, 30)
    g = si.erdos_renyi_gnp(n, 0.3, 9)
    x = np.zeros(n)
    t3, t4 = th["theta3"].astype(np.float64), th["theta4"].astype(np.float64)
    # non-negative weights: relu(theta4 * sum w) == sum relu(theta4 * w)  (Alg. 1 lines 7-8 == Eq. 1)
    g.w = np.abs(si.signed_edge_weights(g, 2, 1.0))
    mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, 1)
    row_sum = si.dense_weights(g).sum(1)
    np.testing.assert_allclose(mu, relu(relu(np.outer(row_sum, t4)) @ t3.T), rtol=1e-12, atol=1e-15)
    # signed weights: the oracle follows Eq. (1) (per-edge relu), which splits by sign of w
    g.w = si.signed_edge_weights(g, 2, 1.0)
    wm = si.dense_weights(g)
    s_pos, s_neg = relu(wm).sum(1), relu(-wm).sum(1)
    e = np.outer(s_pos, relu(t4)) + np.outer(s_neg, relu(-t4))
    mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, 1)
    np.testing.assert_allclose(mu, relu(e @ t3.T), rtol=1e-12, atol=1e-15)
    assert not np.allclose(mu, relu(relu(np.outer(wm.sum(1), t4)) @ t3.T))


# ---- P7: permutation equivariance -------------------------------------------------------

def test_permutation_equivariance(oracle_mod):
    p, T = 6, 3
    th = rand_theta(p, 40)
    g = si.barabasi_albert(60, 3, 11)
    g.w = si.symmetric_edge_weights(g, 5, 0.5, 1.5)
    rng = np.random.default_rng(4)
    x = (rng.random(g.n) < 0.3).astype(np.float64)
    perm = rng.permutation(g.n)
    g2 = si.relabel(g, perm)
    x2 = np.empty_like(x)
    x2[perm] = x
    mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, T)
    mu2 = oracle_mod.embed(g2.rowptr, g2.colidx, g2.w, th, x2, T)
    np.testing.assert_allclose(mu2[perm], mu, rtol=1e-12, atol=1e-14)
    _, q = oracle_mod.q_scores(None, th, mu)
    _, q2 = oracle_mod.q_scores(None, th, mu2)
    np.testing.assert_allclose(q2[perm], q, rtol=1e-12)
    i1, _, _ = oracle_mod.select(None, q, x, None, 1)
    i2, _, _ = oracle_mod.select(None, q2, x2, None, 1)
    assert perm[i1[0, 0]] == i2[0, 0]


# ---- P8: a block-diagonal batch equals its graphs taken alone ------------------------------

def test_batch_equals_single_graphs(oracle_mod):
    p, T = 5, 3
    th = rand_theta(p, 50)
    parts = [si.barabasi_albert(n, 2, s) for n, s in ((13, 1), (30, 2), (5, 3), (21, 4))]
    for i, gpart in enumerate(parts):
        gpart.w = si.symmetric_edge_weights(gpart, 60 + i, 0.5, 1.5)
    batch = si.block_diagonal(parts)
    rng = np.random.default_rng(6)
    x = (rng.random(batch.n) < 0.3).astype(np.float64)
    mu = oracle_mod.embed(batch.rowptr, batch.colidx, batch.w, th, x, T)
    gsum, q = oracle_mod.q_scores(batch.graph_off, th, mu)
    idx, val, cnt = oracle_mod.select(batch.graph_off, q, x, None, 2)
    for b, gpart in enumerate(parts):
        lo, hi = batch.graph_off[b], batch.graph_off[b + 1]
        mu_b = oracle_mod.embed(gpart.rowptr, gpart.colidx, gpart.w, th, x[lo:hi], T)
        assert np.array_equal(mu[lo:hi], mu_b)
        gs_b, q_b = oracle_mod.q_scores(None, th, mu_b)
        assert np.array_equal(gsum[b], gs_b[0]) and np.array_equal(q[lo:hi], q_b)
        i_b, v_b, c_b = oracle_mod.select(None, q_b, x[lo:hi], None, 2)
        assert cnt[b] == c_b[0]
        assert np.array_equal(idx[b][: cnt[b]], i_b[0][: cnt[b]] + lo)
        assert np.array_equal(val[b], v_b[0])


# ---- P10: the graph term of Eq. (2) is constant per graph ----------------------------------

def test_argmax_invariant_to_graph_term(oracle_mod):
    p, T = 6, 3
    th = rand_theta(p, 70)
    g = si.erdos_renyi_gnp(40, 0.2, 13)
    x = (np.random.default_rng(8).random(g.n) < 0.2).astype(np.float64)
    mu = oracle_mod.embed(g.rowptr, g.colidx, None, th, x, T)
    _, q = oracle_mod.q_scores(None, th, mu)
    th2 = dict(th)
    th2["theta6"] = rand_theta(p, 71)["theta6"]
    t5 = th["theta5"].copy()
    t5[:p] = rand_theta(p, 72)["theta5"][:p]
    th2["theta5"] = t5
    _, q2 = oracle_mod.q_scores(None, th2, mu)
    d = q2 - q
    assert np.ptp(d) < 1e-12 * max(1.0, np.abs(q).max()) and abs(d[0]) > 1e-6
    assert oracle_mod.select(None, q, x, None, 5)[0].tolist() == oracle_mod.select(None, q2, x, None, 5)[0].tolist()


# ---- P11: selection against a library sort; d = 1 is the argmax ----------------------------

def test_select_against_lexsort(oracle_mod):
    rng = np.random.default_rng(9)
    n = 500
    q = np.round(rng.normal(size=n), 1)  # many exact ties
    x = (rng.random(n) < 0.3).astype(np.float64)
    cand_idx = np.flatnonzero(x == 0)
    order = cand_idx[np.lexsort((cand_idx, -q[cand_idx]))]
    for k in (1, 7, 64, len(cand_idx), len(cand_idx) + 10):
        idx, val, cnt = oracle_mod.select(None, q, x, None, k)
        take = min(k, len(cand_idx))
        assert cnt[0] == take
        assert np.array_equal(idx[0, :take], order[:take])
        assert np.array_equal(val[0, :take], q[order[:take]])
        assert (idx[0, take:] == -1).all() and np.isneginf(val[0, take:]).all()
    # explicit candidate mask overrides x
    cand = (rng.random(n) < 0.5).astype(np.uint8)
    ci = np.flatnonzero(cand)
    idx, _, _ = oracle_mod.select(None, q, x, cand, 9)
    assert np.array_equal(idx[0], ci[np.lexsort((ci, -q[ci]))][:9])
    # k = 1 is Alg. 3's argmax (lowest index among equal maxima)
    best = cand_idx[q[cand_idx] == q[cand_idx].max()].min()
    assert oracle_mod.select(None, q, x, None, 1)[0][0, 0] == best
    # no candidates at all
    idx, val, cnt = oracle_mod.select(None, q, np.ones(n), None, 3)
    assert cnt[0] == 0 and (idx == -1).all()


# ---- P12: gradients ----------------------------------------------------------------------

def _loss_only(oracle_mod, g, th, x, T, action, target):
    total = 0.0
    S = x.shape[0]
    for b in range(S):
        mu = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x[b], T)
        _, q = oracle_mod.q_scores(g.graph_off, th, mu)
        total += (q[action[b]] - target[b]) ** 2 / S
    return total


def _small_training_case(seed, batched=False):
    if batched:
        parts = [si.erdos_renyi_gnp(6, 0.6, seed), si.erdos_renyi_gnp(5, 0.7, seed + 1)]
        g = si.block_diagonal(parts)
    else:
        g = si.erdos_renyi_gnp(9, 0.4, seed)
    g.w = si.signed_edge_weights(g, seed, 1.0)
    rng = np.random.default_rng(seed)
    S = 3
    x = (rng.random((S, g.n)) < 0.3).astype(np.float64)
    action = rng.integers(0, g.n, size=S).astype(np.int32)
    target = rng.normal(size=S)
    return g, x, action, target


@pytest.mark.parametrize("batched", [False, True])
def test_gradient_vs_central_differences(oracle_mod, batched):
    p, T = 4, 3
    g, x, action, target = _small_training_case(22, batched)
    th = {k: v.astype(np.float64) for k, v in rand_theta(p, 84, std=0.5).items()}
    loss, qp, grads = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, th, x, T, action, target)
    assert abs(loss - _loss_only(oracle_mod, g, th, x, T, action, target)) < 1e-12 * max(1.0, loss)
    h = 1e-6
    for name in si.THETA_NAMES:
        flat = th[name].reshape(-1)
        num = np.zeros_like(flat)
        for i in range(flat.size):
            keep = flat[i]
            flat[i] = keep + h
            lp = _loss_only(oracle_mod, g, th, x, T, action, target)
            flat[i] = keep - h
            lm = _loss_only(oracle_mod, g, th, x, T, action, target)
            flat[i] = keep
            num[i] = (lp - lm) / (2 * h)
        got = grads[name].reshape(-1)
        assert np.abs(got).max() > 0, name
        np.testing.assert_allclose(got, num, rtol=2e-5, atol=2e-7 * max(1.0, np.abs(num).max()), err_msg=name)


def test_gradient_vs_torch_autograd_dense(oracle_mod):
    torch = pytest.importorskip("torch")
    p, T = 4, 4
    g, x, action, target = _small_training_case(33)
    th = {k: v.astype(np.float64) for k, v in rand_theta(p, 81, std=0.4).items()}
    loss, _, grads = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, x, T, action, target)
    th_t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in th.items()}
    adj = torch.tensor(si.dense_adjacency(g))
    wm = torch.tensor(si.dense_weights(g))
    lt = dr.loss_torch(adj, wm, th_t, torch.tensor(x), T, action, torch.tensor(target))
    lt.backward()
    assert abs(float(lt) - loss) < 1e-12 * max(1.0, loss)
    for name in si.THETA_NAMES:
        np.testing.assert_allclose(grads[name], th_t[name].grad.numpy(), rtol=1e-10, atol=1e-13, err_msg=name)


def test_gradient_on_asymmetric_pattern(oracle_mod):
    # The oracle's adjoint of the neighbour sum uses the explicit transpose, so it is right
    # for a directed pattern too; torch autograd on the dense (asymmetric) matrix pins that.
    torch = pytest.importorskip("torch")
    p, T, n = 3, 3, 7
    rng = np.random.default_rng(5)
    dense = (rng.random((n, n)) < 0.4) & ~np.eye(n, dtype=bool)
    rowptr = np.concatenate([[0], np.cumsum(dense.sum(1))]).astype(np.int32)
    colidx = np.concatenate([np.flatnonzero(r) for r in dense]).astype(np.int32)
    w = rng.normal(size=colidx.size)
    wm = np.zeros((n, n))
    wm[dense] = w
    x = rng.normal(size=(2, n))
    action = np.array([1, 4], dtype=np.int32)
    target = rng.normal(size=2)
    th = {k: v.astype(np.float64) for k, v in rand_theta(p, 82, std=0.5).items()}
    loss, _, grads = oracle_mod.loss_grad(rowptr, colidx, w, None, th, x, T, action, target)
    th_t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in th.items()}
    lt = dr.loss_torch(torch.tensor(dense.astype(np.float64)), torch.tensor(wm), th_t, torch.tensor(x), T,
                       action, torch.tensor(target))
    lt.backward()
    assert abs(float(lt) - loss) < 1e-12 * max(1.0, loss)
    for name in si.THETA_NAMES:
        np.testing.assert_allclose(grads[name], th_t[name].grad.numpy(), rtol=1e-10, atol=1e-13, err_msg=name)


def test_sgd_step_decreases_loss_to_first_order(oracle_mod):
    # Sec. 4.5.2: repeated gradient-descent iterations on one minibatch.
    p, T = 4, 3
    g, x, action, target = _small_training_case(44)
    th = {k: v.astype(np.float64) for k, v in rand_theta(p, 83, std=0.4).items()}
    l0, _, grads = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, x, T, action, target)
    lr = 1e-7
    th1 = oracle_mod.sgd(th, grads, lr)
    for k in si.THETA_NAMES:
        np.testing.assert_array_equal(th1[k], th[k] - lr * grads[k])
    l1 = _loss_only(oracle_mod, g, th1, x, T, action, target)
    gnorm2 = sum(float((v ** 2).sum()) for v in grads.values())
    assert l1 < l0
    assert abs((l0 - l1) - lr * gnorm2) < 1e-3 * lr * gnorm2


def test_adjoint_identity_of_neighbour_sum():
    # <A u, v> = <u, A v> on the symmetric CSR the library requires (transpose SpMM == SpMM).
    g = si.barabasi_albert(50, 3, 2)
    adj = si.dense_adjacency(g)
    rng = np.random.default_rng(0)
    u, v = rng.normal(size=g.n), rng.normal(size=g.n)
    assert abs((adj @ u) @ v - u @ (adj @ v)) < 1e-10


# ---- generators ---------------------------------------------------------------------------

def test_generators_produce_valid_symmetric_csr():
    for g in (si.erdos_renyi_gnp(200, 0.05, 1), si.erdos_renyi_gnm(500, 3000, 2), si.barabasi_albert(300, 4, 3),
              si.config(2).graph):
        assert g.rowptr[0] == 0 and g.rowptr[-1] == g.nnz and (np.diff(g.rowptr) >= 0).all()
        rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
        assert (rows != g.colidx).all()
        keys = rows.astype(np.int64) * g.n + g.colidx
        assert (np.diff(keys) > 0).all()  # sorted within rows, no duplicates
        assert np.array_equal(np.sort(g.colidx.astype(np.int64) * g.n + rows), keys)  # symmetric
    g = si.config(2).graph
    w = g.w
    wm = {}
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    for r, c, ww in zip(rows[:2000], g.colidx[:2000], w[:2000]):
        wm[(r, c)] = ww
    for (r, c), ww in wm.items():
        if (c, r) in wm:
            assert wm[(c, r)] == ww
    assert 0.5 <= w.min() and w.max() <= 1.5


def test_barabasi_albert_is_heavy_tailed():
    g = si.barabasi_albert(20000, 8, 5)
    d = g.degrees()
    assert 15.5 < d.mean() < 16.0 and d.max() > 20 * d.mean() and np.median(d) < d.mean()


# ---- Adam and the deep-Q target ------------------------------------------------------------------

def test_adam_matches_torch_optim(oracle_mod):
    # the optimiser of Sec. 4.4, against the library implementation (float64, three steps)
    torch = pytest.importorskip("torch")
    p = 4
    theta = {k: v.astype(np.float64) for k, v in rand_theta(p, 90).items()}
    params = {k: torch.tensor(v.copy(), dtype=torch.float64, requires_grad=True) for k, v in theta.items()}
    opt = torch.optim.Adam(list(params.values()), lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    m = {k: np.zeros_like(v) for k, v in theta.items()}
    v2 = {k: np.zeros_like(v) for k, v in theta.items()}
    for step in (1, 2, 3):
        grads = {k: g.astype(np.float64) for k, g in rand_theta(p, 91 + step, std=1.0).items()}
        for k in params:
            params[k].grad = torch.tensor(grads[k])
        opt.step()
        theta, m, v2 = oracle_mod.adam(theta, grads, m, v2, step, 1e-2)
        for k in params:
            np.testing.assert_allclose(theta[k], params[k].detach().numpy(), rtol=1e-12, atol=1e-15, err_msg=k)


def test_q_target_special_cases(oracle_mod):
    rng = np.random.default_rng(12)
    parts = [si.edgeless(n) for n in (6, 9, 4)]
    g = si.block_diagonal(parts)
    S = 5
    q = rng.normal(size=(S, g.n))
    x = (rng.random((S, g.n)) < 0.4).astype(np.float64)
    action = np.array([0, 7, 16, 3, 10], dtype=np.int32)
    reward = rng.normal(size=S)
    # gamma = 0: the target is the reward
    np.testing.assert_array_equal(oracle_mod.q_target(g.graph_off, q, x, None, action, reward, 0.0), reward)
    # it agrees with the selection routine's best candidate of the action's graph (k = 1)
    t = oracle_mod.q_target(g.graph_off, q, x, None, action, reward, 0.9)
    for b in range(S):
        idx, val, cnt = oracle_mod.select(g.graph_off, q[b], x[b], None, 1)
        gi = int(np.searchsorted(g.graph_off, action[b], side="right") - 1)
        want = reward[b] + (0.9 * val[gi, 0] if cnt[gi] else 0.0)
        assert t[b] == want
    # a state with no candidate in its graph keeps the bare reward
    x[2, g.graph_off[2]:g.graph_off[3]] = 1.0
    assert oracle_mod.q_target(g.graph_off, q, x, None, action, reward, 0.9)[2] == reward[2]
    # an explicit candidate mask overrides x
    cand = np.zeros((S, g.n), np.uint8)
    cand[:, 1] = 1
    t = oracle_mod.q_target(g.graph_off, q, x, cand, np.zeros(S, np.int32), reward, 0.5)
    np.testing.assert_allclose(t, reward + 0.5 * q[:, 1], rtol=0, atol=0)


# ---- weighted neighbour sum: the other reading of the aggregation step of Alg. 1 -----------------

@pytest.mark.parametrize("n,prob,seed", [(8, 0.5, 1), (23, 0.3, 2), (64, 0.2, 3)])
def test_weighted_sum_against_dense_weighted_adjacency(oracle_mod, n, prob, seed):
    # Alg. 1 multiplies the embeddings by the adjacency matrix; with the weights stored in it the
    # neighbour sum is W @ mu.  Dense brute force with that matrix, edge term unchanged.
    p, T = 7, 4
    th = rand_theta(p, 40 + seed)
    g = si.erdos_renyi_gnp(n, prob, seed)
    g.w = si.signed_edge_weights(g, seed, 1.5)
    x = np.random.default_rng(seed).normal(size=n)
    adj, wm = si.dense_adjacency(g), si.dense_weights(g)
    mu, hist = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, T, history=True, weighted=True)
    want, want_hist = dr.embed_dense(adj, wm, th, x, T, history=True, agg=adj * wm)
    for t in range(T):
        np.testing.assert_allclose(hist[t], want_hist[t], rtol=1e-11, atol=1e-13)
    plain = oracle_mod.embed(g.rowptr, g.colidx, g.w, th, x, T)
    assert np.abs(mu - plain).max() > 1e-3          # the two readings really differ on these inputs


def test_weighted_sum_special_weights(oracle_mod):
    p, T = 5, 3
    th = rand_theta(p, 61)
    g = si.erdos_renyi_gnp(30, 0.2, 6)
    x = np.random.default_rng(6).normal(size=g.n)
    # all weights 1 (given or implied): both readings coincide exactly
    ones = np.ones(g.colidx.shape[0])
    a = oracle_mod.embed(g.rowptr, g.colidx, ones, th, x, T, weighted=True)
    assert np.array_equal(a, oracle_mod.embed(g.rowptr, g.colidx, ones, th, x, T))
    assert np.array_equal(a, oracle_mod.embed(g.rowptr, g.colidx, None, th, x, T, weighted=True))
    # all weights c: the weighted sum is c times the plain one, i.e. the plain reading with c * theta2
    c = 2.5
    cw = np.full(g.colidx.shape[0], c)
    th_c = dict(th)
    th_c["theta2"] = th["theta2"].astype(np.float64) * c
    np.testing.assert_allclose(oracle_mod.embed(g.rowptr, g.colidx, cw, th, x, T, weighted=True),
                               oracle_mod.embed(g.rowptr, g.colidx, cw, th_c, x, T), rtol=1e-13, atol=1e-15)


def test_weighted_sum_gradient_vs_torch_autograd_dense(oracle_mod):
    torch = pytest.importorskip("torch")
    p, T = 4, 4
    g, x, action, target = _small_training_case(35)
    th = {k: v.astype(np.float64) for k, v in rand_theta(p, 82, std=0.4).items()}
    loss, _, grads = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, x, T, action, target, weighted=True)
    th_t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in th.items()}
    adj = torch.tensor(si.dense_adjacency(g))
    wm = torch.tensor(si.dense_weights(g))
    lt = dr.loss_torch(adj, wm, th_t, torch.tensor(x), T, action, torch.tensor(target), agg=adj * wm)
    lt.backward()
    assert abs(float(lt) - loss) < 1e-12 * max(1.0, loss)
    for name in si.THETA_NAMES:
        assert np.abs(grads[name]).max() > 0, name
        np.testing.assert_allclose(grads[name], th_t[name].grad.numpy(), rtol=1e-10, atol=1e-13, err_msg=name)
    plain = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, None, th, x, T, action, target)[2]
    assert np.abs(plain["theta2"] - grads["theta2"]).max() > 1e-6
