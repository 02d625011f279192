"""Parity of gradients at relu switches: the oracle's gradient on the branch a float32 evaluation took.

The gradient of Eq. 1 / Eq. 2 jumps wherever a pre-activation crosses zero.  A float32 evaluation (the HIP
path, or any other) resolves the sign of a pre-activation z only when |z| exceeds its own rounding error, a few
float32 roundings of the summed magnitude of z's terms; on a unit inside that band it may take the other
branch than float64, and its gradient then differs from the oracle's by the size of the jump, however
accurate it is.  Instead of avoiding such inputs, the tests read the float32 path's decisions off its
activations, require that they differ from the definition's ONLY inside the band (reported by the oracle
for every unit), and compare the gradient with the oracle's evaluation of that branch
(oracle.loss_grad_decided), at the usual 1e-4.
"""
from __future__ import annotations

import numpy as np

import synth_inputs as si

# A float32 evaluation resolves the sign of a pre-activation z only when |z| exceeds its own rounding error,
# which is a few float32 roundings (2^-24 each) of the summed magnitude of the terms of z.
SIGN_BAND = 1e-6


def decided_reference(oracle, g: si.Graph, theta: dict, x, T: int, action, target, on, on_head=None,
                      weighted: bool = False, band: float = SIGN_BAND, max_open: int = 6):
    """The oracle's gradient on the branch a float32 evaluation took.

    on [S][T][n][p] (bool): that evaluation's relu decisions of Eq. 1, read off its activations.  Every unit
    where they differ from the float64 definition must have |z| <= band * (summed magnitude of the terms of
    z); those units are handed to the oracle as decided.  on_head [S][2][p] likewise for Eq. 2; when it is
    None (the evaluation's head decisions cannot be seen) every head unit inside the band is open, and all
    combinations of the open units are returned (at most 2^max_open).
    Returns (list of (loss, q_pred, grads), info) with info = dict(flips, worst_ratio, open_head)."""
    S, n = np.asarray(x).reshape(-1, g.n).shape
    _, _, _, pre = oracle.loss_grad_decided(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target,
                                            weighted=weighted)
    z, zs, h, hs = pre["z"], pre["zs"], pre["h"], pre["hs"]
    on = np.asarray(on, dtype=bool).reshape(z.shape)
    diff = on != (z > 0)
    ratio = np.abs(z[diff]) / np.maximum(zs[diff], 1e-300)
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= band, f"a relu of Eq. 1 was decided differently although |z| / sum|terms| = {worst:.2e}"
    force = np.full(z.shape, -1, dtype=np.int8)
    force[diff] = on[diff].astype(np.int8)
    fh = np.full(h.shape, -1, dtype=np.int8)
    open_units = []
    if on_head is not None:
        on_head = np.asarray(on_head, dtype=bool).reshape(h.shape)
        dh = on_head != (h > 0)
        rh = np.abs(h[dh]) / np.maximum(hs[dh], 1e-300)
        assert rh.size == 0 or rh.max() <= band, f"a relu of Eq. 2 was decided differently at ratio {rh.max():.2e}"
        fh[dh] = on_head[dh].astype(np.int8)
    else:
        open_units = [tuple(i) for i in np.argwhere(np.abs(h) <= band * hs)]
        assert len(open_units) <= max_open, "too many undecidable head units"
    outs = []
    for combo in range(1 << len(open_units)):
        f2 = fh.copy()
        for k, idx in enumerate(open_units):
            f2[idx] = (combo >> k) & 1
        need = diff.any() or (f2 >= 0).any()
        l, q, gr, _ = oracle.loss_grad_decided(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target,
                                               weighted=weighted, force=force if need else None,
                                               force_head=f2 if need else None)
        outs.append((l, q, gr))
    return outs, dict(flips=int(diff.sum()), worst_ratio=worst, open_head=len(open_units), h=h)


def q_pred_error(theta: dict, h: np.ndarray, got, ref) -> float:
    """Error of the predicted Q of each state's action.  Q is a signed sum of 2p terms theta5_i relu(h_i)
    (Eq. 2) and can be far smaller than they are; its float32 rounding error follows the terms, so each
    state's denominator is floored with 1e-2 of sum_i |theta5_i| relu(h_i), h [S][2][p] from the oracle."""
    t5 = np.abs(np.asarray(theta["theta5"], dtype=np.float64))
    p = t5.shape[0] // 2
    terms = np.maximum(h[:, 0, :], 0.0) @ t5[:p] + np.maximum(h[:, 1, :], 0.0) @ t5[p:]
    ref = np.asarray(ref, dtype=np.float64)
    den = np.maximum(np.abs(ref), np.maximum(1e-2 * terms, 1e-30))
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref) / den))
