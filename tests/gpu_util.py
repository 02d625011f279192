"""Helpers for the GPU parity tests: run the HIP path through the C interface on numpy
inputs and hand back numpy outputs; error metrics used by the parity bars."""
from __future__ import annotations

import numpy as np

import synth_inputs as si


class Device:
    """One context + uploaded graph + workspace, reused across calls of a test."""

    def __init__(self, g: si.Graph, p: int, T: int, S: int = 1, k_max: int = 1, training: bool = False,
                 state_residual: bool = False, weighted_sum: bool = False):
        import torch

        import paper_2105_08764_amd as s2v

        self.torch, self.s2v = torch, s2v
        dev = "cuda"
        self.ctx = s2v.Context()
        self.g_np = g
        self.p, self.T, self.S = p, T, S
        self.graph = s2v.Graph(
            torch.from_numpy(g.rowptr).to(dev),
            torch.from_numpy(g.colidx).to(dev),
            None if g.w is None else torch.from_numpy(g.w).to(dev),
            None if g.graph_off is None else torch.from_numpy(g.graph_off).to(dev),
            state_residual=state_residual, weighted_sum=weighted_sum,
        )
        nbytes = self.ctx.s2v_workspace_bytes(self.graph, p, T, S, k_max, training)
        self.ws_bytes = nbytes
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        assert self.ws.data_ptr() % 256 == 0
        self.ctx.s2v_graph_prepare(self.graph, self.ws)

    def params(self, theta: dict):
        return self.s2v.Params.from_numpy(theta)

    def forward(self, theta, x, save=False):
        """x: float32 [S][N].  Returns dict(mu [N][S][p], gsum [S][G][p], q [S][N], saved or None)."""
        torch = self.torch
        g = self.g_np
        N, G, p, T, S = g.n, g.n_graphs, self.p, self.T, self.S
        prm = theta if isinstance(theta, self.s2v.Params) else self.params(theta)
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32).reshape(S, N)).cuda()
        mu = torch.full((N, S, p), float("nan"), device="cuda")
        saved = torch.full((T, N, S, p), float("nan"), device="cuda") if save else None
        gsum = torch.full((S, G, p), float("nan"), device="cuda")
        q = torch.full((S, N), float("nan"), device="cuda")
        self.ctx.s2v_embed_fwd(self.graph, prm, xd, T, S, mu, saved, gsum, self.ws)
        self.ctx.s2v_q_score(self.graph, prm, mu, gsum, S, q, self.ws)
        torch.cuda.synchronize()
        self.last = dict(x=xd, mu=mu, saved=saved, gsum=gsum, q=q, prm=prm)
        return dict(mu=mu.cpu().numpy(), gsum=gsum.cpu().numpy(), q=q.cpu().numpy(),
                    saved=None if saved is None else saved.cpu().numpy())

    def select(self, q, x, cand, k):
        """q, x: float32 [N]; returns idx [G][k], val [G][k], count [G]."""
        torch = self.torch
        G = self.g_np.n_graphs
        qd = torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).cuda()
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        cd = None if cand is None else torch.from_numpy(np.ascontiguousarray(cand, dtype=np.uint8)).cuda()
        idx = torch.full((G, k), -7, dtype=torch.int32, device="cuda")
        val = torch.full((G, k), float("nan"), device="cuda")
        cnt = torch.full((G,), -7, dtype=torch.int32, device="cuda")
        self.ctx.s2v_select_topk(self.graph, qd, xd, cd, k, idx, val, cnt, self.ws)
        torch.cuda.synchronize()
        return idx.cpu().numpy(), val.cpu().numpy(), cnt.cpu().numpy()

    def train_iter(self, prm, x, action, target, lr=None):
        """One forward + backward (+ SGD step when lr is given) on device parameters prm."""
        torch = self.torch
        g = self.g_np
        N, G, p, T, S = g.n, g.n_graphs, self.p, self.T, self.S
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32).reshape(S, N)).cuda()
        saved = torch.full((T, N, S, p), float("nan"), device="cuda")
        gsum = torch.full((S, G, p), float("nan"), device="cuda")
        ad = torch.from_numpy(np.ascontiguousarray(action, dtype=np.int32)).cuda()
        td = torch.from_numpy(np.ascontiguousarray(target, dtype=np.float32)).cuda()
        loss = torch.full((1,), float("nan"), device="cuda")
        qp = torch.full((S,), float("nan"), device="cuda")
        grads = self.s2v.Params(p, {k: torch.full_like(v, float("nan")) for k, v in prm.t.items()})
        self.ctx.s2v_embed_fwd(self.graph, prm, xd, T, S, None, saved, gsum, self.ws)
        self.ctx.s2v_embed_bwd(self.graph, prm, xd, T, S, saved, gsum, ad, td, loss, qp, grads, self.ws)
        if lr is not None:
            self.ctx.s2v_sgd_step(prm, grads, lr)
        torch.cuda.synchronize()
        self.last_gsum = gsum.cpu().numpy()
        self.last_saved = saved      # [T][N][S][p] on the device: the activations the backward pass read
        return float(loss.item()), qp.cpu().numpy(), grads.to_numpy()

    def last_decisions(self):
        """The relu decisions of the last train_iter as [S][T][N][p] booleans (activation > 0)."""
        return (self.last_saved > 0).permute(2, 0, 1, 3).contiguous().cpu().numpy()


    def loss_grad(self, prm, x, action, target):
        """Forward + backward through the single-call entry point.  Returns (loss, q_pred, grads, gsum)."""
        torch = self.torch
        g = self.g_np
        N, G, p, T, S = g.n, g.n_graphs, self.p, self.T, self.S
        xd = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32).reshape(S, N)).cuda()
        saved = torch.full((T, N, S, p), float("nan"), device="cuda")
        gsum = torch.full((S, G, p), float("nan"), device="cuda")
        ad = torch.from_numpy(np.ascontiguousarray(action, dtype=np.int32)).cuda()
        td = torch.from_numpy(np.ascontiguousarray(target, dtype=np.float32)).cuda()
        loss = torch.full((1,), float("nan"), device="cuda")
        qp = torch.full((S,), float("nan"), device="cuda")
        grads = self.s2v.Params(p, {k: torch.full_like(v, float("nan")) for k, v in prm.t.items()})
        self.ctx.s2v_loss_grad(self.graph, prm, xd, T, S, saved, gsum, ad, td, loss, qp, grads, self.ws)
        torch.cuda.synchronize()
        return float(loss.item()), qp.cpu().numpy(), grads.to_numpy(), gsum.cpu().numpy()


FLOOR_FRAC = 1e-2


def q_term_scale(theta: dict, gsum: np.ndarray, mu: np.ndarray) -> float:
    """Magnitude of the summed terms of Eq. 2 for one state of one graph: sum_i |theta5_i| * relu(.)_i,
    the graph half plus the largest node half.  Q is a signed sum of 2p such terms and can be a
    hundred times smaller than they are; its float32 rounding error follows the terms, so a parity
    check of Q on inputs where that happens floors its denominator with this scale."""
    th = {k: np.asarray(v, dtype=np.float64) for k, v in theta.items()}
    p = th["theta1"].shape[0]
    a = np.abs(th["theta5"][:p]) @ np.maximum(th["theta6"] @ gsum, 0.0)
    b = np.maximum(mu @ th["theta7"].T, 0.0) @ np.abs(th["theta5"][p:])
    return float(a + (b.max() if b.size else 0.0))


def rel_err(got: np.ndarray, ref: np.ndarray, floor_frac: float = FLOOR_FRAC, whole: bool = False,
            scale: float = 0.0) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, floor_frac * max|ref| over the last axis).
    whole=True takes the maximum over the whole array instead (gradient tensors: every entry
    is a sum over the same nodes, states and rounds, so the scale is common to the tensor).

    Plain relative error for every entry that is not small against its own row (a node's
    embedding vector, a graph's sum, a row of a gradient matrix; the whole array for 1-D
    data).  All entries of such a row are sums of terms of one common magnitude, which the
    row's largest entry tracks; an entry far below it is what is left after those terms
    cancelled and carries their absolute float32 rounding error (about p * 2^-24 of the row
    scale), so it is measured against floor_frac * rowmax instead of against itself."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.isfinite(got).all(), "non-finite values in the GPU result"
    rowmax = np.abs(ref).max() if whole else np.abs(ref).max(axis=-1, keepdims=True)
    rowmax = np.maximum(rowmax, scale)       # scale: magnitude of the terms the entries were summed from
    den = np.maximum(np.abs(ref), np.maximum(floor_frac * rowmax, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def rel_err_rms_floor(got: np.ndarray, ref: np.ndarray, floor_frac: float = 1e-3) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, floor_frac * rms(ref)): the stricter reading of "max relative error"
    near cancelled entries (floor at a thousandth of the tensor's root mean square instead of a hundredth of
    the row's maximum).  Reported beside rel_err by the full-size tests; not a bar of its own."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(floor_frac * rms, 1e-30))
    return float(np.max(np.abs(got - ref) / den))


def thetas_clear_of_kinks(oracle, g: si.Graph, p: int, T: int, x, action, target, seed: int, scale: float,
                          eps: float = 2.5e-7, limit: float = 2e-5, tries: int = 24, grad_fn=None):
    """Parameters for a gradient parity case, drawn so that the comparison with float64 is meaningful.

    The gradient of Eq. 1 jumps wherever a pre-activation crosses zero.  With some 10^6 pre-activations
    per case a few always lie within float32 rounding of zero; when one of them also carries a large
    share of the gradient, float32 and float64 take different sides of the relu and the two gradients
    differ by 1e-3 whatever the kernel does.  The float64 oracle shows such a point by itself: along a
    line theta * (1 + k * eps * r), r a random direction and eps four float32 roundings, its gradient
    is smooth (second differences of order eps^2) unless a jump lies on the line, in which case a second
    difference has the size of the jump.  The seeds seed, seed + 1000, ... are tried in order and the
    first is taken for which no second difference over k = -2..2 along three directions exceeds `limit`
    (measured like rel_err over the whole tensor); only the oracle is consulted.
    grad_fn(theta) -> gradient dict replaces the plain oracle call (weighted sum, per-state residual graphs).
    Returns (theta, seed used)."""
    rng = np.random.default_rng(12345)

    def grad(th):
        if grad_fn is not None:
            return grad_fn(th)
        return oracle.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, th, x, T, action, target)[2]

    for k in range(tries):
        sd = seed + 1000 * k
        theta = si.thetas(p, sd, scale)
        ref = grad(theta)
        den = {n: np.maximum(np.abs(ref[n]), max(FLOOR_FRAC * float(np.abs(ref[n]).max()), 1e-30)) for n in si.THETA_NAMES}
        worst = 0.0
        for _ in range(3):
            r = {n: rng.standard_normal(v.shape) for n, v in theta.items()}
            line = [ref if j == 0 else grad({n: v.astype(np.float64) * (1.0 + j * eps * r[n]) for n, v in theta.items()})
                    for j in (-2, -1, 0, 1, 2)]
            for j in (1, 2, 3):
                for n in si.THETA_NAMES:
                    dd = np.abs(line[j - 1][n] - 2.0 * line[j][n] + line[j + 1][n]) / den[n]
                    worst = max(worst, float(dd.max()))
        if worst <= limit:
            return theta, sd
        print(f"theta seed {sd}: the oracle's gradient jumps by {worst:.1e} within {eps:g} of it, skipped", flush=True)
    raise AssertionError("no parameter draw clear of relu kinks found")


def oracle_forward(oracle, g: si.Graph, theta, x_row, T):
    mu = oracle.embed(g.rowptr, g.colidx, g.w, theta, x_row, T)
    gsum, q = oracle.q_scores(g.graph_off, theta, mu)
    return mu, gsum, q


def oracle_per_state_residual(oracle, g: si.Graph, theta, x, T, action=None, target=None, weighted=False):
    """Alg. 4's minibatch on per-state sub-graphs, composed from the oracle's own pieces: state b is
    embedded and scored on residual_graph(x[b]) as a batch of one; with action/target the loss and the
    gradients are the means over the states.  Returns dict(mu [N][S][p], gsum [S][G][p], q [S][N])
    and, when training, (loss, q_pred [S], grads)."""
    S = x.shape[0]
    mus, gsums, qs, losses, qps, gsumd = [], [], [], [], [], None
    for b in range(S):
        rp, ci, w = oracle.residual_graph(g.rowptr, g.colidx, g.w, x[b])
        mu = oracle.embed(rp, ci, w, theta, x[b], T, weighted=weighted)
        gs, q = oracle.q_scores(g.graph_off, theta, mu)
        mus.append(mu.reshape(g.n, -1))
        gsums.append(gs.reshape(g.n_graphs, -1))
        qs.append(q.reshape(-1))
        if action is not None:
            lb, qb, gb = oracle.loss_grad(rp, ci, w, g.graph_off, theta, x[b], T, action[b:b + 1], target[b:b + 1],
                                         weighted=weighted)
            losses.append(lb)
            qps.append(qb[0])
            gsumd = gb if gsumd is None else {k: gsumd[k] + gb[k] for k in gb}
    fwd = dict(mu=np.stack(mus, axis=1), gsum=np.stack(gsums, axis=0), q=np.stack(qs, axis=0))
    if action is None:
        return fwd
    return fwd, (float(np.mean(losses)), np.array(qps), {k: v / S for k, v in gsumd.items()})


def check_selection_with_margin(idx_gpu, cnt_gpu, q_oracle, cand_mask, k, band_rel=1e-4):
    """End-to-end selection check against float64 oracle scores: the GPU's choice must agree
    with the oracle's wherever the oracle's scores are separated by more than the band."""
    cand = np.flatnonzero(cand_mask)
    order = cand[np.lexsort((cand, -q_oracle[cand]))]
    take = min(k, len(cand))
    assert cnt_gpu == take
    if take == 0:
        return 0
    sel = idx_gpu[:take]
    assert len(set(sel.tolist())) == take and cand_mask[sel].all()
    qk = q_oracle[order[take - 1]]
    band = band_rel * max(abs(qk), 1e-30)
    must = order[: take][q_oracle[order[:take]] > qk + band]
    assert np.isin(must, sel).all(), "a clearly-better oracle node is missing from the GPU selection"
    assert (q_oracle[sel] >= qk - band).all(), "the GPU selected a clearly-worse node"
    # positions: exact wherever both neighbours in the oracle order are further away than the band
    exact = 0
    qs = q_oracle[order[:take]]
    for i in range(take):
        left_ok = i == 0 or qs[i - 1] - qs[i] > band
        right_ok = (i == take - 1 and (take == len(order) or qs[i] - q_oracle[order[take]] > band)) or (
            i < take - 1 and qs[i] - qs[i + 1] > band)
        if left_ok and right_ok:
            assert sel[i] == order[i]
            exact += 1
    return exact
