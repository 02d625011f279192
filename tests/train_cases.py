"""The gradient parity cases of tests/test_gpu_train.py: graphs, inputs and the list of (p, T, S),
in a module of their own so that the script that stores their parameter seeds
(tests/golden/make_train_theta_seeds.py, oracle only) builds exactly the same inputs."""
import os

import synth_inputs as si

KINDS = ("er", "ba", "batch")
SHAPES = ((64, 4, 3), (32, 3, 1), (64, 1, 2), (32, 2, 16), (64, 2, 5), (64, 4, 16), (32, 5, 16), (32, 3, 32))
SEED_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "train_theta_seeds.txt")


def graph(kind, seed):
    if kind == "er":
        g = si.erdos_renyi_gnp(300, 0.05, seed)
        g.w = si.signed_edge_weights(g, seed, 1.0)
    elif kind == "ba":
        g = si.barabasi_albert(1500, 4, seed)
        g.w = si.symmetric_edge_weights(g, seed, 0.5, 1.5)
    elif kind == "batch":
        parts = [si.barabasi_albert(n, 2, seed + i) if n > 2 else si.edgeless(n)
                 for i, n in enumerate((40, 1, 77, 1300, 64))]
        g = si.block_diagonal(parts)
    else:
        raise ValueError(kind)
    return g


def inputs(kind, S):
    """Graph, solution flags x [S][N], one action and one target per (state, graph)."""
    g = graph(kind, 3)
    x = si.node_flags(g.n, 0.15, 8, n_states=S)
    action, target = si.training_batch(x, 21)
    return g, x, action, target


def theta_scale(kind):
    return 0.1 if kind != "ba" else 0.05


def first_seed(p, T):
    return 77 + p + T


def stored_seeds():
    out = {}
    with open(SEED_FILE) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                out[(line[0], int(line[1]), int(line[2]), int(line[3]))] = int(line[4])
    return out
