"""The seeded random cases of tests/test_gpu_sweep.py and their oracle side, in a module of their own so that
the script that stores their parameter seeds (tests/golden/make_sweep_theta_seeds.py, oracle only) builds
exactly the same inputs."""
import os

import numpy as np

import synth_inputs as si
from tests import gpu_util as gu

N_CASES = 36
SEED_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "sweep_theta_seeds.txt")


def draw(case):
    rng = np.random.default_rng(9000 + case)
    p = int(rng.choice([32, 64]))
    T = int(rng.integers(1, 6))
    S = int(rng.choice([1, 2, 3, 7, 16, 17, 32, 48]))
    kind = str(rng.choice(["er_sparse", "er_mid", "ba", "star_mix", "batch", "isolated"]))
    weights = str(rng.choice(["unit", "positive", "signed"]))
    weighted_sum = bool(rng.integers(0, 2)) and weights != "unit"
    residual = bool(rng.integers(0, 2))
    xprob = float(rng.choice([0.0, 0.05, 0.3, 0.8]))
    seed = int(rng.integers(1, 1000))
    if kind == "er_sparse":
        g = si.erdos_renyi_gnp(int(rng.integers(40, 500)), 0.03, seed)
    elif kind == "er_mid":
        g = si.erdos_renyi_gnp(int(rng.integers(130, 190)), 0.5, seed)        # rows of two chunks
    elif kind == "ba":
        g = si.barabasi_albert(int(rng.integers(100, 600)), int(rng.integers(1, 6)), seed)
    elif kind == "star_mix":
        g = si.block_diagonal([si.star_graph(int(rng.integers(300, 900))), si.erdos_renyi_gnp(60, 0.2, seed)])
        g = si.Graph(g.n, g.rowptr, g.colidx, None, None)                     # one graph with a long row
    elif kind == "batch":
        parts = [si.barabasi_albert(int(n), 2, seed + i) if n > 2 else si.edgeless(int(n))
                 for i, n in enumerate(rng.integers(1, 200, size=int(rng.integers(2, 7))))]
        g = si.block_diagonal(parts)
    else:
        g = si.block_diagonal([si.edgeless(int(rng.integers(1, 40))), si.erdos_renyi_gnp(80, 0.1, seed)])
        g = si.Graph(g.n, g.rowptr, g.colidx, None, None)                     # isolated nodes in front
    if weights == "positive":
        g.w = si.symmetric_edge_weights(g, seed, 0.5, 1.5)
    elif weights == "signed":
        g.w = si.signed_edge_weights(g, seed, 1.0)
    deg = max(1.0, g.nnz / max(g.n, 1))
    scale = float(min(0.1, 0.6 / np.sqrt(deg * p)))     # keeps the rounds from growing by more than ~x2 each
    x = si.node_flags(g.n, xprob, seed + 1, n_states=S)
    desc = f"p={p} T={T} S={S} {kind} n={g.n} nnz={g.nnz} G={g.n_graphs} w={weights} wsum={weighted_sum} res={residual} x={xprob}"
    return dict(p=p, T=T, S=S, g=g, x=x, weighted_sum=weighted_sum, residual=residual, scale=scale, seed=seed, desc=desc)


def oracle_forward(oracle, c, theta):
    g, x, T = c["g"], c["x"], c["T"]
    if c["residual"]:
        return gu.oracle_per_state_residual(oracle, g, theta, x, T, weighted=c["weighted_sum"])
    mus, gss, qs = [], [], []
    for b in range(c["S"]):
        mu = oracle.embed(g.rowptr, g.colidx, g.w, theta, x[b], T, weighted=c["weighted_sum"])
        gs, q = oracle.q_scores(g.graph_off, theta, mu)
        mus.append(mu.reshape(g.n, -1)); gss.append(gs.reshape(g.n_graphs, -1)); qs.append(q.reshape(-1))
    return dict(mu=np.stack(mus, axis=1), gsum=np.stack(gss, axis=0), q=np.stack(qs, axis=0))


def training_inputs(c):
    """x (every state with a node outside its solution), actions, targets of case c."""
    x = c["x"].copy()
    if (x == 0).sum(axis=1).min() == 0:
        x[:, 0] = 0
    action, target = si.training_batch(x, c["seed"] + 3)
    return x, action, target


def oracle_loss_grad(oracle, c, theta, x, action, target):
    g, T = c["g"], c["T"]
    if c["residual"]:
        return gu.oracle_per_state_residual(oracle, g, theta, x, T, action, target, weighted=c["weighted_sum"])[1]
    return oracle.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target,
                            weighted=c["weighted_sum"])


def first_theta_seed(c):
    return c["seed"] + 11


def screened_theta(oracle, c, x, action, target):
    """First parameter draw of case c without a relu switch within float32 rounding (oracle only)."""
    return gu.thetas_clear_of_kinks(oracle, c["g"], c["p"], c["T"], x, action, target, first_theta_seed(c), c["scale"],
                                    grad_fn=lambda th: oracle_loss_grad(oracle, c, th, x, action, target)[2])


def stored_seeds():
    out = {}
    with open(SEED_FILE) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[int(line[0])] = int(line[1])
    return out


def q_pred_scales(oracle, c, theta, x, action):
    """Per state: the magnitude of the terms that Eq. 2 sums at the action node (gu.q_term_scale), from the
    oracle's forward pass; the float32 error of the predicted Q follows it, not Q itself."""
    ref = oracle_forward(oracle, dict(c, x=x), theta)
    offs = c["g"].offsets()
    out = []
    for b in range(c["S"]):
        a = int(action[b])
        gi = int(np.searchsorted(offs, a, side="right") - 1)
        out.append(gu.q_term_scale(theta, ref["gsum"][b, gi], ref["mu"][a:a + 1, b, :]))
    return np.array(out)
