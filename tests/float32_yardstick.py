"""A plain float32 evaluation of the training step (Train of Alg. 4: Eq. 1, Eq. 2, squared loss, reverse
mode) that shares nothing with the HIP kernels: dense adjacency matrices and torch CPU autograd.

It is a yardstick, not a reference.  The gradient of Eq. 1 jumps wherever a pre-activation crosses zero; a
float32 evaluation and the float64 oracle take different sides of such a relu whenever the pre-activation
lies within float32 rounding of zero, and then differ by the size of the jump whatever the implementation.
How often that happens on a family of inputs is a property of float32 arithmetic on those inputs; this
module measures it, so that the HIP path's miss rate has something to be compared with.
"""
from __future__ import annotations

import numpy as np

import synth_inputs as si


def loss_grad_float32(g: si.Graph, theta: dict, x: np.ndarray, T: int, action, target, weighted: bool = False,
                      decisions: bool = False):
    """(loss, q_pred [S], grads dict) in float32 on the dense form of Eq. 1 / Eq. 2.
    The graph sum of Eq. 2 runs over the graph (of a block-diagonal batch) that holds the state's action.
    decisions=True appends (on [S][T][n][p], on_head [S][2][p]): which relu units passed their input."""
    import torch

    dt = torch.float32
    n = g.n
    adj = torch.tensor(si.dense_adjacency(g), dtype=dt)
    wm = torch.tensor(si.dense_weights(g), dtype=dt)
    th = {k: torch.tensor(np.asarray(v), dtype=dt, requires_grad=True) for k, v in theta.items()}
    p = th["theta1"].shape[0]
    agg = adj * wm if weighted else adj
    off = np.array([0, n]) if g.graph_off is None else np.asarray(g.graph_off)
    xs = torch.tensor(np.asarray(x).reshape(-1, n), dtype=dt)
    S = xs.shape[0]
    # third term of Eq. 1: the same for every state and round
    e = (adj[:, :, None] * torch.relu(wm[:, :, None] * th["theta4"][None, None, :])).sum(dim=1)
    edge = e @ th["theta3"].T
    total = torch.zeros((), dtype=dt)
    qs = []
    on = np.zeros((S, T, n, p), dtype=bool)
    on_head = np.zeros((S, 2, p), dtype=bool)
    for b in range(S):
        const = torch.outer(xs[b], th["theta1"]) + edge
        mu = torch.zeros(n, p, dtype=dt)
        for t in range(T):
            mu = torch.relu(const + (agg @ mu) @ th["theta2"].T)
            on[b, t] = mu.detach().numpy() > 0
        a = int(action[b])
        gi = int(np.searchsorted(off, a, side="right") - 1)
        gs = mu[int(off[gi]):int(off[gi + 1])].sum(dim=0)
        h1, h2 = th["theta6"] @ gs, th["theta7"] @ mu[a]
        on_head[b, 0], on_head[b, 1] = h1.detach().numpy() > 0, h2.detach().numpy() > 0
        q = th["theta5"][:p] @ torch.relu(h1) + th["theta5"][p:] @ torch.relu(h2)
        qs.append(float(q.detach()))
        total = total + (q - float(np.float32(target[b]))) ** 2 / S
    total.backward()
    out = (float(total.detach()), np.array(qs), {k: v.grad.numpy().astype(np.float64) for k, v in th.items()})
    return out + (on, on_head) if decisions else out


def worst_gradient_error(got: dict, ref: dict, floor_frac: float = 1e-2) -> float:
    """The parity metric of the gradient tests (tests/gpu_util.rel_err with whole=True), worst tensor."""
    worst = 0.0
    for name in si.THETA_NAMES:
        r = np.asarray(ref[name], dtype=np.float64)
        d = np.abs(np.asarray(got[name], dtype=np.float64) - r)
        den = np.maximum(np.abs(r), max(floor_frac * float(np.abs(r).max()), 1e-30))
        worst = max(worst, float((d / den).max()))
    return worst

