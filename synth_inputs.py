"""Seeded synthetic inputs for the structure2vec / deep-Q hot path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
bench.  It holds graph generators, CSR packing and random draws only: none of
the method's arithmetic (no embedding, scoring, selection or gradient code).

Workloads follow the graph families the paper evaluates on (Sec. 6.1:
Erdos-Renyi and Barabasi-Albert random graphs) at the shapes named by the
benchmark configurations.  All randomness comes from numpy PCG64 generators
with explicit seeds, or from a counter-based hash for per-edge weights.

Conventions
-----------
* CSR is symmetric (each undirected edge stored twice), int32, rows sorted by
  column, no duplicates, no self-loops.
* Every float input is drawn in float64 and rounded to float32; the GPU takes
  the float32 array, the oracle takes the same values widened to float64.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np


@dataclass
class Graph:
    """Symmetric CSR graph, optionally a block-diagonal batch of graphs."""

    n: int
    rowptr: np.ndarray  # int32 [n+1]
    colidx: np.ndarray  # int32 [nnz]
    w: Optional[np.ndarray] = None  # float32 [nnz] or None (all 1.0)
    graph_off: Optional[np.ndarray] = None  # int32 [G+1] or None (G == 1)

    @property
    def nnz(self) -> int:
        return int(self.colidx.shape[0])

    @property
    def n_graphs(self) -> int:
        return 1 if self.graph_off is None else int(self.graph_off.shape[0] - 1)

    def offsets(self) -> np.ndarray:
        if self.graph_off is None:
            return np.array([0, self.n], dtype=np.int32)
        return self.graph_off

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr)


# ----------------------------------------------------------------------------
# CSR packing
# ----------------------------------------------------------------------------

def csr_from_undirected(n: int, a: np.ndarray, b: np.ndarray) -> Graph:
    """Pack undirected edges {a_i, b_i} into a symmetric, sorted, deduplicated CSR."""
    a = np.asarray(a, dtype=np.int64)
    b = np.asarray(b, dtype=np.int64)
    keep = a != b
    a, b = a[keep], b[keep]
    keys = np.concatenate([a * n + b, b * n + a])
    del a, b
    keys.sort()
    if keys.size:
        uniq = np.empty(keys.shape, dtype=bool)
        uniq[0] = True
        np.not_equal(keys[1:], keys[:-1], out=uniq[1:])
        keys = keys[uniq]
        del uniq
    rows = keys // n
    cols = (keys - rows * n).astype(np.int32)
    del keys
    counts = np.bincount(rows, minlength=n)
    del rows
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2**31
    return Graph(n=n, rowptr=rowptr.astype(np.int32), colidx=cols)


def dense_adjacency(g: Graph) -> np.ndarray:
    """0/1 float64 adjacency matrix (small graphs only; used by brute-force pins)."""
    adj = np.zeros((g.n, g.n), dtype=np.float64)
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    adj[rows, g.colidx] = 1.0
    return adj


def dense_weights(g: Graph) -> np.ndarray:
    """Float64 matrix of edge weights (0 where there is no edge)."""
    wm = np.zeros((g.n, g.n), dtype=np.float64)
    rows = np.repeat(np.arange(g.n), np.diff(g.rowptr))
    wm[rows, g.colidx] = 1.0 if g.w is None else g.w.astype(np.float64)
    return wm


# ----------------------------------------------------------------------------
# Graph families
# ----------------------------------------------------------------------------

def erdos_renyi_gnp(n: int, prob: float, seed: int) -> Graph:
    """G(n, p): every unordered pair independently with probability prob (O(n^2), small n)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    iu, ju = np.triu_indices(n, k=1)
    pick = rng.random(iu.shape[0]) < prob
    return csr_from_undirected(n, iu[pick], ju[pick])


def erdos_renyi_gnm(n: int, m_edges: int, seed: int) -> Graph:
    """G(n, M) stand-in for G(n, p) at large n: M uniformly random pairs, O(M).

    Self-pairs and repeated pairs are dropped, so the edge count is M minus a
    handful (expected about M^2 / n^2 repeats)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.integers(0, n, size=m_edges, dtype=np.int64)
    b = rng.integers(0, n, size=m_edges, dtype=np.int64)
    return csr_from_undirected(n, a, b)


def barabasi_albert(n: int, m: int, seed: int) -> Graph:
    """Preferential attachment: each new vertex attaches m edges to endpoints drawn
    uniformly from the endpoint list of all earlier edges (Batagelj-Brandes list
    method), starting from a star on vertices 0..m.  Repeated targets of one new
    vertex collapse to one edge, so degrees are >= 1 and mostly >= m."""
    assert n > m >= 1
    rng = np.random.Generator(np.random.PCG64(seed))
    n_new = n - m - 1  # vertices m+1 .. n-1 attach preferentially
    n_edges = m * (n - m)
    src = np.empty(n_edges, dtype=np.int64)
    src[:m] = m
    if n_new > 0:
        src[m:] = np.repeat(np.arange(m + 1, n, dtype=np.int64), m)
    # ref[e] = position in the endpoint list (2*e' = source of e', 2*e'+1 = target of e')
    # that edge e copies its target from; seed edges have explicit targets.
    ref = np.full(n_edges, -1, dtype=np.int64)
    if n_new > 0:
        earlier = 2 * m * (np.repeat(np.arange(m + 1, n, dtype=np.int64), m) - m)
        ref[m:] = np.minimum((rng.random(n_edges - m) * earlier).astype(np.int64), earlier - 1)
    tgt = np.full(n_edges, -1, dtype=np.int64)
    tgt[:m] = np.arange(m)
    # Resolve references by pointer jumping: an even position names a source vertex
    # directly; an odd position forwards to the reference of that earlier edge.
    pending = np.arange(m, n_edges)
    cur = ref[m:].copy()
    while pending.size:
        even = (cur & 1) == 0
        e_ref = cur >> 1
        done_even = even
        tgt[pending[done_even]] = src[e_ref[done_even]]
        odd_idx = ~even
        tgt_known = tgt[e_ref] >= 0
        done_odd = odd_idx & tgt_known
        tgt[pending[done_odd]] = tgt[e_ref[done_odd]]
        still = odd_idx & ~tgt_known
        # forward the reference one hop
        nxt = ref[e_ref[still]]
        pending = pending[still]
        cur = nxt
    assert (tgt >= 0).all()
    return csr_from_undirected(n, src, tgt)


def block_diagonal(graphs: Sequence[Graph]) -> Graph:
    """Pack independent graphs into one block-diagonal CSR with per-graph node offsets."""
    sizes = np.array([g.n for g in graphs], dtype=np.int64)
    off = np.zeros(len(graphs) + 1, dtype=np.int64)
    np.cumsum(sizes, out=off[1:])
    rowptr = [np.zeros(1, dtype=np.int64)]
    colidx = []
    ws = []
    base = 0
    for g, o in zip(graphs, off[:-1]):
        rowptr.append(g.rowptr[1:].astype(np.int64) + base)
        colidx.append(g.colidx.astype(np.int64) + o)
        if g.w is not None:
            ws.append(g.w)
        base += g.nnz
    has_w = len(ws) == len(graphs) and len(graphs) > 0
    return Graph(
        n=int(off[-1]),
        rowptr=np.concatenate(rowptr).astype(np.int32),
        colidx=(np.concatenate(colidx).astype(np.int32) if colidx else np.zeros(0, np.int32)),
        w=(np.concatenate(ws).astype(np.float32) if has_w else None),
        graph_off=off.astype(np.int32),
    )


def cycle_graph(n: int) -> Graph:
    a = np.arange(n)
    return csr_from_undirected(n, a, (a + 1) % n)


def complete_graph(n: int) -> Graph:
    iu, ju = np.triu_indices(n, k=1)
    return csr_from_undirected(n, iu, ju)


def star_graph(n_leaves: int) -> Graph:
    """Vertex 0 is the hub; vertices 1..n_leaves are leaves."""
    return csr_from_undirected(n_leaves + 1, np.zeros(n_leaves, dtype=np.int64), np.arange(1, n_leaves + 1))


def complete_bipartite(a: int, b: int) -> Graph:
    left = np.repeat(np.arange(a), b)
    right = a + np.tile(np.arange(b), a)
    return csr_from_undirected(a + b, left, right)


def edgeless(n: int) -> Graph:
    return Graph(n=n, rowptr=np.zeros(n + 1, dtype=np.int32), colidx=np.zeros(0, dtype=np.int32))


def relabel(g: Graph, perm: np.ndarray) -> Graph:
    """Graph with node v renamed perm[v] (weights follow their edges)."""
    rows = np.repeat(np.arange(g.n, dtype=np.int64), np.diff(g.rowptr))
    r2 = perm[rows].astype(np.int64)
    c2 = perm[g.colidx].astype(np.int64)
    order = np.argsort(r2 * g.n + c2, kind="stable")
    counts = np.bincount(r2, minlength=g.n)
    rowptr = np.zeros(g.n + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    return Graph(
        n=g.n,
        rowptr=rowptr.astype(np.int32),
        colidx=c2[order].astype(np.int32),
        w=None if g.w is None else g.w[order],
        graph_off=None,
    )


# ----------------------------------------------------------------------------
# Random draws
# ----------------------------------------------------------------------------

def _splitmix64(z: np.ndarray) -> np.ndarray:
    z = (z + np.uint64(0x9E3779B97F4A7C15)).astype(np.uint64)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def symmetric_edge_weights(g: Graph, seed: int, lo: float, hi: float) -> np.ndarray:
    """float32 weight per stored entry, equal for (v,u) and (u,v): U(lo, hi) keyed on the
    unordered pair through a counter-based hash, so no sort is needed."""
    rows = np.repeat(np.arange(g.n, dtype=np.uint64), np.diff(g.rowptr))
    cols = g.colidx.astype(np.uint64)
    a = np.minimum(rows, cols)
    b = np.maximum(rows, cols)
    with np.errstate(over="ignore"):
        h = _splitmix64(_splitmix64(a * np.uint64(g.n) + b) ^ np.uint64(seed))
    u = (h >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return (lo + (hi - lo) * u).astype(np.float32)


def signed_edge_weights(g: Graph, seed: int, scale: float = 1.0) -> np.ndarray:
    """Symmetric weights of both signs, U(-scale, scale); only for tests of the edge term."""
    return symmetric_edge_weights(g, seed, -scale, scale)


THETA_NAMES = ("theta1", "theta2", "theta3", "theta4", "theta5", "theta6", "theta7")


def theta_shapes(p: int) -> dict:
    """Shapes in the library's numbering; 4p^2 + 4p values in total (Sec. 5.1 item 3)."""
    return {
        "theta1": (p,),
        "theta2": (p, p),
        "theta3": (p, p),
        "theta4": (p,),
        "theta5": (2 * p,),
        "theta6": (p, p),
        "theta7": (p, p),
    }


def thetas(p: int, seed: int, std: float = 0.1) -> dict:
    """theta_i ~ N(0, std^2), float32, row-major [out][in] for the matrices."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return {k: (rng.standard_normal(s) * std).astype(np.float32) for k, s in theta_shapes(p).items()}


def node_flags(n: int, prob: float, seed: int, n_states: int = 1) -> np.ndarray:
    """x[s][v] ~ Bernoulli(prob) as float32 0/1 (the partial-solution indicator)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.random((n_states, n)) < prob).astype(np.float32)


def training_batch(x: np.ndarray, seed: int, g: Optional[Graph] = None):
    """One action node per state, uniform over that state's nodes with x == 0, and a
    target value ~ N(0, 1) (float32)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n_states = x.shape[0]
    action = np.empty(n_states, dtype=np.int32)
    for s in range(n_states):
        free = np.flatnonzero(x[s] == 0)
        action[s] = free[rng.integers(0, free.shape[0])]
    target = rng.standard_normal(n_states).astype(np.float32)
    return action, target


# ----------------------------------------------------------------------------
# The five benchmark configurations
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    graph: Graph
    p: int
    T: int
    theta: dict
    x: np.ndarray  # float32 [S][N]
    k: int  # nodes to select per graph (1 = argmax)
    action: Optional[np.ndarray] = None  # int32 [S]
    target: Optional[np.ndarray] = None  # float32 [S]
    lr: float = 0.0
    iters: int = 0


def _one_percent_k(x_row: np.ndarray) -> int:
    return max(1, int(0.01 * int((x_row == 0).sum())))


def config(c: int, scale: float = 1.0) -> Workload:
    """Benchmark configuration c in 1..5 (6 = the paper's own ER(21000, 0.15) shape).  scale < 1
    shrinks the node count of the large configurations for quick parity runs; the structure is
    unchanged."""
    gs, xs, ts, ws, trs = 1000 + c, 2000 + c, 3000 + c, 4000 + c, 5000 + c
    if c == 1:
        g = erdos_renyi_gnp(1000, 0.01, gs)
        x = node_flags(g.n, 0.1, xs)
        return Workload("cfg1_er1k", g, 32, 3, thetas(32, ts), x, 1)
    if c == 2:
        parts = [barabasi_albert(500, 4, gs * 1000 + i) for i in range(128)]
        g = block_diagonal(parts)
        g.w = symmetric_edge_weights(g, ws, 0.5, 1.5)
        x = node_flags(g.n, 0.2, xs)
        return Workload("cfg2_ba500x128", g, 64, 4, thetas(64, ts), x, 1)
    if c in (3, 5):
        n = max(64, int(round(1_000_000 * scale)))
        g = barabasi_albert(n, 8, 1003)
        if c == 3:
            x = node_flags(g.n, 0.05, xs)
            return Workload("cfg3_ba1m", g, 64, 4, thetas(64, ts), x, _one_percent_k(x[0]))
        x = node_flags(g.n, 0.05, xs, n_states=16)
        action, target = training_batch(x, trs)
        return Workload("cfg5_train_ba1m", g, 64, 4, thetas(64, ts), x, 1,
                        action=action, target=target, lr=1e-3, iters=4)
    if c == 4:
        n = max(64, int(round(2_000_000 * scale)))
        g = erdos_renyi_gnm(n, 15 * n, gs)
        g.w = symmetric_edge_weights(g, ws, 0.5, 1.5)
        x = node_flags(g.n, 0.05, xs)
        return Workload("cfg4_er2m", g, 64, 4, thetas(64, ts), x, _one_percent_k(x[0]))
    if c == 6:
        # The paper's own large test shape (Sec. 6.4): Erdos-Renyi, 21 000 nodes, edge probability
        # 0.15 (about 33 million edges, average degree 3 150), K = 32, L = 2.  G(n, M) stands in for
        # G(n, p); M = -ln(1 - p) * C(n, 2) random pairs leave p * C(n, 2) distinct ones on average.
        n = max(64, int(round(21_000 * scale)))
        g = erdos_renyi_gnm(n, int(-np.log(1.0 - 0.15) * n * (n - 1) / 2), gs)
        x = node_flags(g.n, 0.05, xs)
        return Workload("cfg6_paper_er21k", g, 32, 2, thetas(32, ts), x, 1)
    raise ValueError(f"no such configuration: {c}")
