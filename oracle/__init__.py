"""TEST INFRASTRUCTURE: ctypes front end of the float64 CPU oracle (oracle/s2v_oracle.c).

Only tests, the smoke check and the bench's cpu_baseline leg may import this package.
It is independent of the HIP library: it shares no code with it and neither imports
the other.  Inputs are numpy arrays; float inputs of any precision are widened to
float64 before the C code sees them.

Functions mirror the C entry points: embed (Eq. 1 / Alg. 1), q_scores (Eq. 2 / Alg. 2),
select (Alg. 3's argmax and the top-d selection of Sec. 4.5.1), loss_grad (the Train
step of Alg. 4; loss_grad_decided: the same with relu decisions given by the caller) and sgd (plain gradient descent, repeated as in Sec. 4.5.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "s2v_oracle.c")
_LIB = os.path.join(_HERE, "libs2v_oracle.so")

THETA_NAMES = ("theta1", "theta2", "theta3", "theta4", "theta5", "theta6", "theta7")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2 + OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"], cwd=_HERE
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _th(theta: dict):
    return [_f64(theta[k]) for k in THETA_NAMES]


def embed(rowptr, colidx, w, theta: dict, x, T: int, history: bool = False, weighted: bool = False):
    """mu^T as [n][p] float64 (and mu^1..mu^T as [T][n][p] when history is set).
    weighted: the neighbour sum of Eq. 1 weights neighbour u of v by w(v, u)."""
    lib = _load()
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.shape[0] - 1
    th = _th(theta)
    p = th[0].shape[0]
    wd = None if w is None else _f64(w)
    xd = _f64(x).reshape(-1)
    assert xd.shape[0] == n
    mu = np.zeros((n, p), dtype=np.float64)
    hist = np.zeros((T, n, p), dtype=np.float64) if history else None
    rc = lib.oracle_embed(
        ctypes.c_int32(n), _ptr(rowptr), _ptr(colidx), _ptr(wd), ctypes.c_int32(int(bool(weighted))),
        ctypes.c_int32(p), ctypes.c_int32(T),
        _ptr(th[0]), _ptr(th[1]), _ptr(th[2]), _ptr(th[3]), _ptr(xd), _ptr(mu), _ptr(hist),
    )
    assert rc == 0
    return (mu, hist) if history else mu


def q_scores(graph_off, theta: dict, mu):
    """(gsum [G][p], q [n]) for a block-diagonal batch; graph_off None means one graph."""
    lib = _load()
    mu = _f64(mu)
    n, p = mu.shape
    th = _th(theta)
    go = None if graph_off is None else _i32(graph_off)
    G = 1 if go is None else go.shape[0] - 1
    gsum = np.zeros((G, p), dtype=np.float64)
    q = np.zeros(n, dtype=np.float64)
    rc = lib.oracle_q(ctypes.c_int32(n), ctypes.c_int32(G), _ptr(go), ctypes.c_int32(p),
                      _ptr(th[4]), _ptr(th[5]), _ptr(th[6]), _ptr(mu), _ptr(gsum), _ptr(q))
    assert rc == 0
    return gsum, q


def select(graph_off, q, x, cand, k: int):
    """(idx [G][k] int32, val [G][k] float64, count [G] int32)."""
    lib = _load()
    q = _f64(q)
    n = q.shape[0]
    xd = _f64(x).reshape(-1)
    go = None if graph_off is None else _i32(graph_off)
    G = 1 if go is None else go.shape[0] - 1
    cd = None if cand is None else np.ascontiguousarray(cand, dtype=np.uint8)
    idx = np.zeros((G, k), dtype=np.int32)
    val = np.zeros((G, k), dtype=np.float64)
    cnt = np.zeros(G, dtype=np.int32)
    rc = lib.oracle_select(ctypes.c_int32(n), ctypes.c_int32(G), _ptr(go), _ptr(q), _ptr(xd), _ptr(cd),
                           ctypes.c_int32(k), _ptr(idx), _ptr(val), _ptr(cnt))
    assert rc == 0
    return idx, val, cnt


def loss_grad(rowptr, colidx, w, graph_off, theta: dict, x, T: int, action, target, weighted: bool = False):
    """(loss, q_pred [S], grads dict) for the squared loss averaged over the S states."""
    lib = _load()
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.shape[0] - 1
    th = _th(theta)
    p = th[0].shape[0]
    wd = None if w is None else _f64(w)
    xd = _f64(x).reshape(-1, n)
    S = xd.shape[0]
    go = None if graph_off is None else _i32(graph_off)
    G = 1 if go is None else go.shape[0] - 1
    act = _i32(action)
    tgt = _f64(target)
    assert act.shape[0] == S and tgt.shape[0] == S
    loss = np.zeros(1, dtype=np.float64)
    qp = np.zeros(S, dtype=np.float64)
    grads = [np.zeros_like(t) for t in th]
    rc = lib.oracle_loss_grad(
        ctypes.c_int32(n), _ptr(rowptr), _ptr(colidx), _ptr(wd), ctypes.c_int32(int(bool(weighted))),
        ctypes.c_int32(G), _ptr(go),
        ctypes.c_int32(p), ctypes.c_int32(T), *[_ptr(t) for t in th], ctypes.c_int32(S), _ptr(xd),
        _ptr(act), _ptr(tgt), _ptr(loss), _ptr(qp), *[_ptr(g) for g in grads],
    )
    assert rc == 0, rc
    return float(loss[0]), qp, dict(zip(THETA_NAMES, grads))


def loss_grad_decided(rowptr, colidx, w, graph_off, theta: dict, x, T: int, action, target, weighted: bool = False,
                      force=None, force_head=None):
    """loss_grad with some relu decisions taken by the caller, plus every pre-activation.

    force: int8 [S][T][n][p] or None, force_head: int8 [S][2][p] or None; -1 = follow the sign of the
    pre-activation, 0 / 1 = unit off / on (Eq. 1 units; Eq. 2 units: row 0 theta6 g, row 1 theta7 mu_action).
    Returns (loss, q_pred, grads, info) with info = dict(z, zs [S][T][n][p], h, hs [S][2][p]): the
    pre-activations and the summed magnitudes of their terms.  With no forced decision the first three
    equal loss_grad's bit for bit."""
    lib = _load()
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.shape[0] - 1
    th = _th(theta)
    p = th[0].shape[0]
    wd = None if w is None else _f64(w)
    xd = _f64(x).reshape(-1, n)
    S = xd.shape[0]
    go = None if graph_off is None else _i32(graph_off)
    G = 1 if go is None else go.shape[0] - 1
    act = _i32(action)
    tgt = _f64(target)
    assert act.shape[0] == S and tgt.shape[0] == S
    fo = None if force is None else np.ascontiguousarray(force, dtype=np.int8)
    fh = None if force_head is None else np.ascontiguousarray(force_head, dtype=np.int8)
    assert fo is None or fo.shape == (S, T, n, p)
    assert fh is None or fh.shape == (S, 2, p)
    loss = np.zeros(1, dtype=np.float64)
    qp = np.zeros(S, dtype=np.float64)
    grads = [np.zeros_like(t) for t in th]
    z = np.zeros((S, T, n, p), dtype=np.float64)
    zs = np.zeros((S, T, n, p), dtype=np.float64)
    h = np.zeros((S, 2, p), dtype=np.float64)
    hs = np.zeros((S, 2, p), dtype=np.float64)
    rc = lib.oracle_loss_grad_decided(
        ctypes.c_int32(n), _ptr(rowptr), _ptr(colidx), _ptr(wd), ctypes.c_int32(int(bool(weighted))),
        ctypes.c_int32(G), _ptr(go),
        ctypes.c_int32(p), ctypes.c_int32(T), *[_ptr(t) for t in th], ctypes.c_int32(S), _ptr(xd),
        _ptr(act), _ptr(tgt), _ptr(loss), _ptr(qp), *[_ptr(g) for g in grads],
        _ptr(fo), _ptr(fh), _ptr(z), _ptr(zs), _ptr(h), _ptr(hs),
    )
    assert rc == 0, rc
    return float(loss[0]), qp, dict(zip(THETA_NAMES, grads)), dict(z=z, zs=zs, h=h, hs=hs)


def sgd(theta: dict, grads: dict, lr: float) -> dict:
    """theta - lr * grad for every parameter, in float64."""
    lib = _load()
    out = {}
    for k in THETA_NAMES:
        t = _f64(theta[k]).copy()
        g = _f64(grads[k])
        lib.oracle_sgd(ctypes.c_int64(t.size), _ptr(t), _ptr(g), ctypes.c_double(lr))
        out[k] = t
    return out


# ---- the inference loop of Alg. 3 with the multiple-node selection of Sec. 4.5.1 ---------------

def residual_graph(rowptr, colidx, w, x):
    """The adjacency structure after Alg. 3's update: every edge with an endpoint in the partial
    solution (x != 0) removed.  Same node set; returns (rowptr, colidx, w) of the remaining edges."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    n = rowptr.shape[0] - 1
    x = _f64(x).reshape(-1)
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    keep = (x[rows] == 0) & (x[colidx] == 0)
    counts = np.bincount(rows[keep], minlength=n)
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(counts, out=rp[1:])
    return rp.astype(np.int32), colidx[keep], (None if w is None else np.asarray(w)[keep])


def adaptive_d(n_candidates: int, n_nodes: int) -> int:
    """Sec. 4.5.1: 8 nodes per evaluation while |C| > N/2, 4 for (N/4, N/2], 2 for (N/8, N/4], else 1."""
    if n_candidates > n_nodes / 2:
        return 8
    if n_candidates > n_nodes / 4:
        return 4
    if n_candidates > n_nodes / 8:
        return 2
    return 1


def mvc_inference(rowptr, colidx, w, graph_off, theta: dict, x, T: int, adaptive: bool, max_steps: int,
                  weighted: bool = False):
    """Alg. 3 for minimum vertex cover, one state: repeat {embed on the remaining graph, score,
    add the d best candidates to the solution} until no edge remains.  Candidates are the nodes
    outside the solution that still have an edge.  Returns (x, steps, trace) with trace a list of
    (d, selected ids, candidates before the step, stored entries left before the step)."""
    x = _f64(x).reshape(-1).copy()
    n = x.shape[0]
    go = None if graph_off is None else _i32(graph_off)
    G = 1 if go is None else go.shape[0] - 1
    trace = []
    steps = 0
    while steps < max_steps:
        rp, ci, ww = residual_graph(rowptr, colidx, w, x)
        live = int(ci.shape[0])
        if live == 0:
            break
        cand = ((x == 0) & (np.diff(rp) > 0)).astype(np.uint8)
        d = adaptive_d(int(cand.sum()), n) if (adaptive and G == 1) else 1
        mu = embed(rp, ci, ww, theta, x, T, weighted=weighted)
        _, q = q_scores(go, theta, mu)
        idx, _, cnt = select(go, q, x, cand, d)
        chosen = np.concatenate([idx[b, : cnt[b]] for b in range(G)])
        trace.append((d, chosen.copy(), int(cand.sum()), live))
        x[chosen] = 1.0
        steps += 1
    return x, steps, trace


# ---- the rest of the paper's Train step: Adam and the deep-Q target ----------------------------

def adam(theta: dict, grads: dict, m: dict, v: dict, step: int, lr: float, beta1=0.9, beta2=0.999, eps=1e-8):
    """One Adam step in float64 (the optimiser of Sec. 4.4): returns new (theta, m, v) dicts."""
    out_t, out_m, out_v = {}, {}, {}
    for k in THETA_NAMES:
        g = _f64(grads[k])
        mk = beta1 * _f64(m[k]) + (1.0 - beta1) * g
        vk = beta2 * _f64(v[k]) + (1.0 - beta2) * g * g
        m_hat = mk / (1.0 - beta1 ** step)
        v_hat = vk / (1.0 - beta2 ** step)
        out_t[k] = _f64(theta[k]) - lr * m_hat / (np.sqrt(v_hat) + eps)
        out_m[k], out_v[k] = mk, vk
    return out_t, out_m, out_v


def q_target(graph_off, q_next, x_next, cand_next, action, reward, gamma: float):
    """target[b] = reward[b] + gamma * (largest next-state score among the candidates of the graph
    that holds action[b]); reward[b] alone when no candidate is left (Alg. 4's target value)."""
    q_next = _f64(q_next)
    S, n = q_next.shape
    x_next = _f64(x_next).reshape(S, n)
    go = np.array([0, n], dtype=np.int32) if graph_off is None else _i32(graph_off)
    out = np.zeros(S, dtype=np.float64)
    for b in range(S):
        gidx = int(np.searchsorted(go, int(action[b]) if action is not None else 0, side="right") - 1)
        lo, hi = int(go[gidx]), int(go[gidx + 1])
        best = None
        for v in range(lo, hi):
            is_c = (cand_next[b][v] != 0) if cand_next is not None else (x_next[b][v] == 0)
            if is_c and (best is None or q_next[b][v] > best):
                best = q_next[b][v]
        out[b] = reward[b] + (gamma * best if best is not None else 0.0)
    return out
