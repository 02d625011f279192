"""Thin Python binding of libs2v.so (the MI355X structure2vec / deep-Q hot path).

Argument marshalling only: every step runs in the library's HIP kernels.  PyTorch is
used for device memory and streams.  The functions carry the names of the C entry
points declared in include/s2v.h and take torch CUDA tensors (float32 / int32 / uint8,
contiguous).  There is no CPU fallback: if the shared library has not been built
(`python -m paper_2105_08764_amd.build`), loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs2v.so")

S2V_OK = 0
SINGLE_LAUNCH_AUTO, SINGLE_LAUNCH_ALWAYS, SINGLE_LAUNCH_NEVER = 0, 1, 2   # modes of s2v_set_single_launch
S2V_ERR_INVALID_ARG = -1
S2V_ERR_UNSUPPORTED = -2
S2V_ERR_WORKSPACE_TOO_SMALL = -3
S2V_ERR_HIP = -4
S2V_ERR_NO_DEVICE = -5
S2V_ERR_NOT_PREPARED = -6
S2V_ERR_TOO_LARGE = -7
S2V_NOALLOC_MAX_NODES = 1 << 22
S2V_NOALLOC_MAX_K = 1 << 18

PROFILE_KINDS = ("fwd_round", "bwd_round", "fwd_round2", "fwd_round_q", "bwd_round_mask", "bwd_first", "bwd_seed",
                 "select")
THETA_NAMES = ("theta1", "theta2", "theta3", "theta4", "theta5", "theta6", "theta7")
EXPORTS = (
    "s2v_status_str", "s2v_create", "s2v_destroy", "s2v_last_hip_error", "s2v_workspace_bytes",
    "s2v_graph_prepare", "s2v_embed_fwd", "s2v_q_score", "s2v_select_topk", "s2v_embed_bwd",
    "s2v_sgd_step", "s2v_adaptive_d", "s2v_profile_begin", "s2v_profile_end", "s2v_residual_update",
    "s2v_mvc_inference", "s2v_adam_step", "s2v_q_target", "s2v_policy_eval", "s2v_loss_grad",
    "s2v_select_topk_noalloc", "s2v_set_sliced_min_bytes", "s2v_set_single_launch", "s2v_stream_read",
    "s2v_policy_select",
)


class S2VError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where}: {text} (status {status})")
        self.status = status


class CGraph(ctypes.Structure):
    _fields_ = [
        ("n_nodes", ctypes.c_int32),
        ("nnz", ctypes.c_int64),
        ("rowptr", ctypes.c_void_p),
        ("colidx", ctypes.c_void_p),
        ("w", ctypes.c_void_p),
        ("n_graphs", ctypes.c_int32),
        ("graph_off", ctypes.c_void_p),
        ("row_end", ctypes.c_void_p),
        ("state_residual", ctypes.c_int32),
        ("weighted_sum", ctypes.c_int32),
    ]


class CParams(ctypes.Structure):
    _fields_ = [("p", ctypes.c_int32)] + [(k, ctypes.c_void_p) for k in THETA_NAMES]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libs2v.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2105_08764_amd.build` "
                "(there is no fallback path)"
            )
        lib = ctypes.CDLL(LIB_PATH)
        lib.s2v_status_str.restype = ctypes.c_char_p
        lib.s2v_status_str.argtypes = [ctypes.c_int32]
        lib.s2v_adaptive_d.restype = ctypes.c_int32
        lib.s2v_adaptive_d.argtypes = [ctypes.c_int64, ctypes.c_int64]
        for name in EXPORTS:
            fn = getattr(lib, name)
            if name not in ("s2v_status_str",):
                fn.restype = ctypes.c_int32
        _lib = lib
    return _lib


def s2v_status_str(status: int) -> str:
    return load_library().s2v_status_str(int(status)).decode()


def s2v_adaptive_d(n_candidates: int, n_nodes: int) -> int:
    return int(load_library().s2v_adaptive_d(int(n_candidates), int(n_nodes)))


def _check(status: int, where: str) -> None:
    if status != S2V_OK:
        raise S2VError(status, where, s2v_status_str(status))


def _dp(t) -> Optional[int]:
    """Device pointer of a tensor (None stays NULL)."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _want(t, dtype, what):
    import torch

    if t is not None and t.dtype != getattr(torch, dtype):
        raise TypeError(f"{what} must be {dtype}, got {t.dtype}")


class Graph:
    """Device-side CSR graph (or block-diagonal batch); keeps the tensors alive."""

    def __init__(self, rowptr, colidx, w=None, graph_off=None, row_end=None, state_residual=False, weighted_sum=False):
        _want(row_end, "int32", "row_end")
        _want(rowptr, "int32", "rowptr")
        _want(colidx, "int32", "colidx")
        _want(w, "float32", "w")
        _want(graph_off, "int32", "graph_off")
        self.rowptr, self.colidx, self.w, self.graph_off, self.row_end = rowptr, colidx, w, graph_off, row_end
        self.n_nodes = int(rowptr.numel() - 1)
        self.nnz = int(colidx.numel())
        self.n_graphs = 1 if graph_off is None else int(graph_off.numel() - 1)
        self.c = CGraph(self.n_nodes, self.nnz, _dp(rowptr), _dp(colidx) if self.nnz else None, _dp(w),
                        self.n_graphs, _dp(graph_off), _dp(row_end), int(bool(state_residual)), int(bool(weighted_sum)))
        self.state_residual = bool(state_residual)
        self.weighted_sum = bool(weighted_sum)

    def mutable_copy(self):
        """A copy whose colidx / w / row_end the inference loop may edit in place."""
        return Graph(self.rowptr, self.colidx.clone(), None if self.w is None else self.w.clone(), self.graph_off,
                     self.rowptr[1:].clone(), state_residual=self.state_residual, weighted_sum=self.weighted_sum)


class Params:
    """The seven parameter tensors on the device (also used for gradients)."""

    def __init__(self, p: int, tensors: dict):
        self.p = int(p)
        self.t = {k: tensors[k] for k in THETA_NAMES}
        for k, v in self.t.items():
            _want(v, "float32", k)
        self.c = CParams(self.p, *[_dp(self.t[k]) for k in THETA_NAMES])

    @staticmethod
    def from_numpy(theta: dict, device="cuda"):
        import torch

        p = int(theta["theta1"].shape[0])
        return Params(p, {k: torch.from_numpy(theta[k]).to(device).contiguous() for k in THETA_NAMES})

    @staticmethod
    def zeros_like(other: "Params"):
        import torch

        return Params(other.p, {k: torch.zeros_like(v) for k, v in other.t.items()})

    def to_numpy(self) -> dict:
        return {k: v.detach().cpu().numpy() for k, v in self.t.items()}


class Context:
    """s2v_ctx bound to a torch stream (default: the current stream at construction)."""

    def __init__(self, stream=None):
        import torch

        self.lib = load_library()
        if not torch.cuda.is_available():
            raise S2VError(S2V_ERR_NO_DEVICE, "Context", "no GPU visible to torch")
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self.handle = ctypes.c_void_p()
        _check(self.lib.s2v_create(ctypes.c_void_p(self.stream.cuda_stream), ctypes.byref(self.handle)), "s2v_create")

    def close(self):
        if self.handle:
            self.lib.s2v_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- one method per C entry point ------------------------------------------------------
    def s2v_workspace_bytes(self, g: Graph, p: int, T: int, S: int, k_max: int, training: bool = False) -> int:
        out = ctypes.c_size_t(0)
        _check(self.lib.s2v_workspace_bytes(self.handle, ctypes.byref(g.c), ctypes.c_int32(p), ctypes.c_int32(T),
                                            ctypes.c_int32(S), ctypes.c_int32(k_max), ctypes.c_int32(int(training)),
                                            ctypes.byref(out)), "s2v_workspace_bytes")
        return int(out.value)

    def s2v_graph_prepare(self, g: Graph, ws) -> None:
        _check(self.lib.s2v_graph_prepare(self.handle, ctypes.byref(g.c), ctypes.c_void_p(_dp(ws)),
                                          ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_graph_prepare")

    def s2v_embed_fwd(self, g: Graph, params: Params, x, T: int, S: int, mu_out, mu_saved, gsum, ws) -> None:
        _want(x, "float32", "x")
        _check(self.lib.s2v_embed_fwd(self.handle, ctypes.byref(g.c), ctypes.byref(params.c), ctypes.c_void_p(_dp(x)),
                                      ctypes.c_int32(T), ctypes.c_int32(S), ctypes.c_void_p(_dp(mu_out)),
                                      ctypes.c_void_p(_dp(mu_saved)), ctypes.c_void_p(_dp(gsum)),
                                      ctypes.c_void_p(_dp(ws)), ctypes.c_size_t(ws.numel() * ws.element_size())),
               "s2v_embed_fwd")

    def s2v_policy_eval(self, g: Graph, params: Params, x, T: int, S: int, mu_out, gsum, q, ws) -> None:
        _want(x, "float32", "x")
        _check(self.lib.s2v_policy_eval(self.handle, ctypes.byref(g.c), ctypes.byref(params.c),
                                        ctypes.c_void_p(_dp(x)), ctypes.c_int32(T), ctypes.c_int32(S),
                                        ctypes.c_void_p(_dp(mu_out)), ctypes.c_void_p(_dp(gsum)),
                                        ctypes.c_void_p(_dp(q)), ctypes.c_void_p(_dp(ws)),
                                        ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_policy_eval")

    def s2v_q_score(self, g: Graph, params: Params, mu, gsum, S: int, q, ws) -> None:
        _check(self.lib.s2v_q_score(self.handle, ctypes.byref(g.c), ctypes.byref(params.c), ctypes.c_void_p(_dp(mu)),
                                    ctypes.c_void_p(_dp(gsum)), ctypes.c_int32(S), ctypes.c_void_p(_dp(q)),
                                    ctypes.c_void_p(_dp(ws)), ctypes.c_size_t(ws.numel() * ws.element_size())),
               "s2v_q_score")

    def s2v_select_topk(self, g: Graph, q, x, cand, k: int, idx, val, count, ws) -> None:
        _want(idx, "int32", "idx")
        _want(count, "int32", "count")
        _want(cand, "uint8", "cand")
        _check(self.lib.s2v_select_topk(self.handle, ctypes.byref(g.c), ctypes.c_void_p(_dp(q)),
                                        ctypes.c_void_p(_dp(x)), ctypes.c_void_p(_dp(cand)), ctypes.c_int32(k),
                                        ctypes.c_void_p(_dp(idx)), ctypes.c_void_p(_dp(val)),
                                        ctypes.c_void_p(_dp(count)), ctypes.c_void_p(_dp(ws)),
                                        ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_select_topk")

    def s2v_policy_select(self, g: Graph, params: Params, x, cand, T: int, k: int, mu_out, gsum, q, idx, val, count,
                          ws) -> None:
        _want(x, "float32", "x")
        _want(idx, "int32", "idx")
        _want(count, "int32", "count")
        _want(cand, "uint8", "cand")
        _check(self.lib.s2v_policy_select(self.handle, ctypes.byref(g.c), ctypes.byref(params.c),
                                          ctypes.c_void_p(_dp(x)), ctypes.c_void_p(_dp(cand)), ctypes.c_int32(T),
                                          ctypes.c_int32(k), ctypes.c_void_p(_dp(mu_out)), ctypes.c_void_p(_dp(gsum)),
                                          ctypes.c_void_p(_dp(q)), ctypes.c_void_p(_dp(idx)), ctypes.c_void_p(_dp(val)),
                                          ctypes.c_void_p(_dp(count)), ctypes.c_void_p(_dp(ws)),
                                          ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_policy_select")

    def s2v_select_topk_noalloc(self, n_nodes: int, q, x, cand, k: int, idx, val, count) -> None:
        _want(idx, "int32", "idx")
        _want(count, "int32", "count")
        _want(cand, "uint8", "cand")
        _check(self.lib.s2v_select_topk_noalloc(self.handle, ctypes.c_int32(n_nodes), ctypes.c_void_p(_dp(q)),
                                                ctypes.c_void_p(_dp(x)), ctypes.c_void_p(_dp(cand)), ctypes.c_int32(k),
                                                ctypes.c_void_p(_dp(idx)), ctypes.c_void_p(_dp(val)),
                                                ctypes.c_void_p(_dp(count))), "s2v_select_topk_noalloc")

    def s2v_embed_bwd(self, g: Graph, params: Params, x, T: int, S: int, mu_saved, gsum, action, target, loss,
                      q_pred, grads: Params, ws) -> None:
        _want(action, "int32", "action")
        _check(self.lib.s2v_embed_bwd(self.handle, ctypes.byref(g.c), ctypes.byref(params.c), ctypes.c_void_p(_dp(x)),
                                      ctypes.c_int32(T), ctypes.c_int32(S), ctypes.c_void_p(_dp(mu_saved)),
                                      ctypes.c_void_p(_dp(gsum)), ctypes.c_void_p(_dp(action)),
                                      ctypes.c_void_p(_dp(target)), ctypes.c_void_p(_dp(loss)),
                                      ctypes.c_void_p(_dp(q_pred)), ctypes.byref(grads.c), ctypes.c_void_p(_dp(ws)),
                                      ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_embed_bwd")

    def s2v_loss_grad(self, g: Graph, params: Params, x, T: int, S: int, mu_saved, gsum, action, target, loss,
                      q_pred, grads: Params, ws) -> None:
        _want(action, "int32", "action")
        _check(self.lib.s2v_loss_grad(self.handle, ctypes.byref(g.c), ctypes.byref(params.c), ctypes.c_void_p(_dp(x)),
                                      ctypes.c_int32(T), ctypes.c_int32(S), ctypes.c_void_p(_dp(mu_saved)),
                                      ctypes.c_void_p(_dp(gsum)), ctypes.c_void_p(_dp(action)),
                                      ctypes.c_void_p(_dp(target)), ctypes.c_void_p(_dp(loss)),
                                      ctypes.c_void_p(_dp(q_pred)), ctypes.byref(grads.c), ctypes.c_void_p(_dp(ws)),
                                      ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_loss_grad")

    def s2v_adam_step(self, params: Params, grads: Params, m: Params, v: Params, step: int, lr: float,
                      beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
        _check(self.lib.s2v_adam_step(self.handle, ctypes.byref(params.c), ctypes.byref(grads.c), ctypes.byref(m.c),
                                      ctypes.byref(v.c), ctypes.c_int32(step), ctypes.c_float(lr),
                                      ctypes.c_float(beta1), ctypes.c_float(beta2), ctypes.c_float(eps)),
               "s2v_adam_step")

    def s2v_q_target(self, g: Graph, q_next, x_next, cand_next, action, reward, gamma: float, S: int, target, ws) -> None:
        _check(self.lib.s2v_q_target(self.handle, ctypes.byref(g.c), ctypes.c_void_p(_dp(q_next)),
                                     ctypes.c_void_p(_dp(x_next)), ctypes.c_void_p(_dp(cand_next)),
                                     ctypes.c_void_p(_dp(action)), ctypes.c_void_p(_dp(reward)),
                                     ctypes.c_float(gamma), ctypes.c_int32(S), ctypes.c_void_p(_dp(target)),
                                     ctypes.c_void_p(_dp(ws)), ctypes.c_size_t(ws.numel() * ws.element_size())),
               "s2v_q_target")

    def s2v_residual_update(self, g: Graph, x, sel_idx, sel_count, k: int, cand, stats, ws) -> None:
        _want(cand, "uint8", "cand")
        _want(stats, "int32", "stats")
        _check(self.lib.s2v_residual_update(self.handle, ctypes.byref(g.c), ctypes.c_void_p(_dp(x)),
                                            ctypes.c_void_p(_dp(sel_idx)), ctypes.c_void_p(_dp(sel_count)),
                                            ctypes.c_int32(k), ctypes.c_void_p(_dp(cand)), ctypes.c_void_p(_dp(stats)),
                                            ctypes.c_void_p(_dp(ws)), ctypes.c_size_t(ws.numel() * ws.element_size())),
               "s2v_residual_update")

    def s2v_mvc_inference(self, g: Graph, params: Params, x, T: int, adaptive: bool, max_steps: int, mu, gsum, q, cand,
                          sel_idx, sel_val, sel_count, stats, ws):
        """Returns (policy evaluations, nodes added, live stored entries left)."""
        steps = ctypes.c_int32(0)
        picked = ctypes.c_int64(0)
        live = ctypes.c_int64(0)
        _check(self.lib.s2v_mvc_inference(self.handle, ctypes.byref(g.c), ctypes.byref(params.c),
                                          ctypes.c_void_p(_dp(x)), ctypes.c_int32(T), ctypes.c_int32(int(adaptive)),
                                          ctypes.c_int32(max_steps), ctypes.c_void_p(_dp(mu)),
                                          ctypes.c_void_p(_dp(gsum)), ctypes.c_void_p(_dp(q)),
                                          ctypes.c_void_p(_dp(cand)), ctypes.c_void_p(_dp(sel_idx)),
                                          ctypes.c_void_p(_dp(sel_val)), ctypes.c_void_p(_dp(sel_count)),
                                          ctypes.c_void_p(_dp(stats)), ctypes.byref(steps), ctypes.byref(picked),
                                          ctypes.byref(live), ctypes.c_void_p(_dp(ws)),
                                          ctypes.c_size_t(ws.numel() * ws.element_size())), "s2v_mvc_inference")
        return int(steps.value), int(picked.value), int(live.value)

    def s2v_profile_begin(self, max_launches: int) -> None:
        _check(self.lib.s2v_profile_begin(self.handle, ctypes.c_int32(max_launches)), "s2v_profile_begin")

    def s2v_profile_end(self):
        """{kind name: (spans, total ms)} for the kinds of include/s2v.h (S2V_PROFILE_*)."""
        n = (ctypes.c_int32 * len(PROFILE_KINDS))()
        ms = (ctypes.c_float * len(PROFILE_KINDS))()
        _check(self.lib.s2v_profile_end(self.handle, n, ms), "s2v_profile_end")
        return {name: (int(n[i]), float(ms[i])) for i, name in enumerate(PROFILE_KINDS)}

    def s2v_set_sliced_min_bytes(self, nbytes: int) -> None:
        _check(self.lib.s2v_set_sliced_min_bytes(self.handle, ctypes.c_size_t(nbytes)), "s2v_set_sliced_min_bytes")

    def s2v_set_single_launch(self, mode: int) -> None:
        _check(self.lib.s2v_set_single_launch(self.handle, ctypes.c_int32(mode)), "s2v_set_single_launch")

    def s2v_stream_read(self, src, out) -> None:
        _check(self.lib.s2v_stream_read(self.handle, ctypes.c_void_p(_dp(src)),
                                        ctypes.c_size_t(src.numel() * src.element_size()),
                                        ctypes.c_void_p(_dp(out))), "s2v_stream_read")

    def s2v_sgd_step(self, params: Params, grads: Params, lr: float) -> None:
        _check(self.lib.s2v_sgd_step(self.handle, ctypes.byref(params.c), ctypes.byref(grads.c), ctypes.c_float(lr)),
               "s2v_sgd_step")
