"""Dense-matrix restatements of Eq. (1) / Eq. (2) used ONLY to pin the CPU oracle.

These are written against the adjacency MATRIX (numpy / torch float64), not against
CSR rows, so they share no indexing logic with the oracle's C loops: a wrong index,
a dropped term or a transposed operand in the oracle shows up as a mismatch here.
"""
import numpy as np


def relu(a):
    return np.maximum(a, 0.0)


def edge_term(adj, wm, th4):
    """e[v][k] = sum_u adj[v][u] * relu(th4[k] * W[v][u])   (third term of Eq. 1, before theta3)."""
    return np.einsum("vu,vuk->vk", adj, relu(wm[:, :, None] * th4[None, None, :]))


def embed_dense(adj, wm, th, x, T, history=False, agg=None):
    """T rounds of Eq. (1) from a zero embedding; rows of MU are nodes.  agg is the matrix of the
    neighbour sum: the 0/1 adjacency (default, Eq. 1 as printed) or the weighted adjacency."""
    agg = adj if agg is None else agg
    th = {k: np.asarray(v, dtype=np.float64) for k, v in th.items()}
    n = adj.shape[0]
    p = th["theta1"].shape[0]
    mu = np.zeros((n, p))
    const = np.outer(x, th["theta1"]) + edge_term(adj, wm, th["theta4"]) @ th["theta3"].T
    hist = []
    for _ in range(T):
        mu = relu(const + (agg @ mu) @ th["theta2"].T)
        hist.append(mu)
    return (mu, hist) if history else mu


def q_dense(th, mu):
    """Eq. (2) for every node of one graph."""
    th = {k: np.asarray(v, dtype=np.float64) for k, v in th.items()}
    p = th["theta1"].shape[0]
    g = mu.sum(axis=0)
    qa = th["theta5"][:p] @ relu(th["theta6"] @ g)
    qb = relu(mu @ th["theta7"].T) @ th["theta5"][p:]
    return qa + qb


def loss_torch(adj, wm, th_t, x_states, T, action, target, agg=None):
    """Squared loss averaged over states, in torch float64 on dense matrices (for autograd)."""
    import torch

    agg = adj if agg is None else agg
    p = th_t["theta1"].shape[0]
    total = 0.0
    S = x_states.shape[0]
    for b in range(S):
        e = (adj[:, :, None] * torch.relu(wm[:, :, None] * th_t["theta4"][None, None, :])).sum(dim=1)
        const = torch.outer(x_states[b], th_t["theta1"]) + e @ th_t["theta3"].T
        mu = torch.zeros(adj.shape[0], p, dtype=torch.float64)
        for _ in range(T):
            mu = torch.relu(const + (agg @ mu) @ th_t["theta2"].T)
        g = mu.sum(dim=0)
        q = th_t["theta5"][:p] @ torch.relu(th_t["theta6"] @ g) + th_t["theta5"][p:] @ torch.relu(
            th_t["theta7"] @ mu[action[b]]
        )
        total = total + (q - target[b]) ** 2 / S
    return total


def loss_torch_decided(adj, wm, th_t, x_states, T, action, target, force, force_head):
    """loss_torch with relu decisions given from outside: force [S][T][n][p] and force_head [S][2][p] hold
    -1 (the unit follows the sign of its pre-activation), 0 (off) or 1 (on: it passes its pre-activation
    whatever its sign).  Pins oracle.loss_grad_decided."""
    import torch

    p = th_t["theta1"].shape[0]
    total = 0.0
    S = x_states.shape[0]

    def act(z, f):
        f = torch.as_tensor(np.asarray(f))
        on = torch.where(f < 0, z.detach() > 0, f > 0)
        return z * on.to(z.dtype)

    for b in range(S):
        e = (adj[:, :, None] * torch.relu(wm[:, :, None] * th_t["theta4"][None, None, :])).sum(dim=1)
        const = torch.outer(x_states[b], th_t["theta1"]) + e @ th_t["theta3"].T
        mu = torch.zeros(adj.shape[0], p, dtype=adj.dtype)
        for t in range(T):
            mu = act(const + (adj @ mu) @ th_t["theta2"].T, force[b][t])
        g = mu.sum(dim=0)
        q = th_t["theta5"][:p] @ act(th_t["theta6"] @ g, force_head[b][0]) + th_t["theta5"][p:] @ act(
            th_t["theta7"] @ mu[action[b]], force_head[b][1])
        total = total + (q - target[b]) ** 2 / S
    return total
