#!/usr/bin/env python3
"""Benchmark of the structure2vec / deep-Q hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-train] [--no-loop] [--no-cpu-baseline]

A "step" is one RL inference step on the 30M-edge workload (benchmark configuration 4:
Erdos-Renyi n = 2e6, average degree 30, p = 64, T = 4): embedding and scores (s2v_policy_eval:
the work of s2v_embed_fwd + s2v_q_score) and top-k selection with k = 1 % of the candidates (s2v_select_topk), with all
inputs resident in HBM.  The one-time graph preparation is timed separately.  Also reported:
the training step of configuration 5 (Barabasi-Albert n = 1e6, 16 states, 4 SGD iterations),
the live HIP-event time of the fused embedding-round kernel against the HBM roofline, and the
float64 CPU oracle timed on the host cores as a baseline.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def round_algorithmic_bytes(n, nnz, p, S=1):
    """Bytes one fused embedding round must move when no gathered row is reused:
    rowptr + colidx + one p-float row per stored entry + x, s+, s- + the output rows."""
    return 4 * (n + 1) + 4 * nnz + 4 * p * nnz * S + 12 * n * S + 4 * p * n * S


def copy_ceiling_gbs(torch):
    """Empirical streaming ceiling of this GPU: a plain 1 GiB device-to-device copy (1 GiB read +
    1 GiB written), best of five, in GB/s of total traffic."""
    src = torch.empty(1 << 28, device="cuda").normal_()
    dst = torch.empty_like(src)
    best = float("inf")
    for _ in range(6):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        dst.copy_(src)
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b))
    del src, dst
    torch.cuda.empty_cache()
    return 2 * (1 << 30) / (best * 1e-3) / 1e9


def read_traffic(path):
    """HBM bytes per launch of the embedding-round kernel from a committed rocprofv3 counter
    summary (FETCH_SIZE + WRITE_SIZE, scaled); None if the summary is not there."""
    try:
        for line in open(path):
            if line.startswith("HBM_BYTES_PER_LAUNCH="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def upload(s2v, torch, g):
    return s2v.Graph(
        torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda(),
        None if g.w is None else torch.from_numpy(g.w).cuda(),
        None if g.graph_off is None else torch.from_numpy(g.graph_off).cuda())


def bench_inference(args, s2v, torch):
    t0 = time.time()
    w = si.config(4, args.scale)
    g = w.graph
    log(f"[bench] config 4 generated: n={g.n} nnz={g.nnz} k={w.k} ({time.time() - t0:.1f}s)")
    ctx = s2v.Context()
    torch.cuda.reset_peak_memory_stats()
    graph = upload(s2v, torch, g)
    prm = s2v.Params.from_numpy(w.theta)
    N, p, T, k = g.n, w.p, w.T, w.k
    ws = torch.empty(ctx.s2v_workspace_bytes(graph, p, T, 1, k), dtype=torch.uint8, device="cuda")
    x = torch.from_numpy(w.x).cuda()
    mu = torch.empty((N, 1, p), device="cuda")
    gsum = torch.empty((1, 1, p), device="cuda")
    q = torch.empty((1, N), device="cuda")
    idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
    val = torch.empty((1, k), device="cuda")
    cnt = torch.empty((1,), dtype=torch.int32, device="cuda")

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.s2v_graph_prepare(graph, ws)
    torch.cuda.synchronize()
    prepare_ms = (time.perf_counter() - t0) * 1e3

    def step():
        ctx.s2v_policy_eval(graph, prm, x, T, 1, mu, gsum, q, ws)      # embedding (Alg. 1) + scores (Alg. 2)
        ctx.s2v_select_topk(graph, q[0], x[0], None, k, idx, val, cnt, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.s2v_profile_begin(args.steps * (T - 1) + 4)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    (n_round, ms_round), _, (n_r2, ms_r2), (n_rq, ms_rq) = ctx.s2v_profile_end()
    peak_mb = torch.cuda.max_memory_allocated() / 2**20
    round_ms = ms_round / max(n_round, 1)
    alg = round_algorithmic_bytes(N, g.nnz, p)
    achieved = alg / (round_ms * 1e-3) / 1e9
    log(f"[bench] inference {ms:.3f} ms/step; round 2 (from scalars) {ms_r2 / max(n_r2, 1):.3f} ms; "
        f"gather round {round_ms:.3f} ms x {n_round}, last round with the node term of Q "
        f"{ms_rq / max(n_rq, 1):.3f} ms x {n_rq}; "
        f"{achieved:.0f} GB/s algorithmic; prepare {prepare_ms:.1f} ms; peak {peak_mb:.0f} MiB")
    # the same step with the weighted neighbour sum (the other reading of Alg. 1's aggregation):
    # each round also reads the 4-byte weight of every stored entry
    graph_w = s2v.Graph(graph.rowptr, graph.colidx, graph.w, graph.graph_off, weighted_sum=True)

    def step_w():
        ctx.s2v_policy_eval(graph_w, prm, x, T, 1, mu, gsum, q, ws)
        ctx.s2v_select_topk(graph_w, q[0], x[0], None, k, idx, val, cnt, ws)

    step_w()
    torch.cuda.synchronize()
    ctx.s2v_profile_begin(3 * (T - 1) + 4)
    t0 = time.perf_counter()
    for _ in range(3):
        step_w()
    torch.cuda.synchronize()
    ms_w = (time.perf_counter() - t0) * 1e3 / 3
    (n_round_w, ms_round_w), _, _, _ = ctx.s2v_profile_end()
    round_w_ms = ms_round_w / max(n_round_w, 1)
    log(f"[bench] weighted neighbour sum: {ms_w:.3f} ms/step, gather round {round_w_ms:.3f} ms "
        f"({(alg + 4 * g.nnz) / (round_w_ms * 1e-3) / 1e9:.0f} GB/s algorithmic)")
    step()      # leave the buffers holding the plain reading's result
    torch.cuda.synchronize()
    out = dict(
        weighted_sum=dict(ms_per_step=ms_w, round_ms=round_w_ms,
                          round_gbs=(alg + 4 * g.nnz) / (round_w_ms * 1e-3) / 1e9),
        ms=ms, prepare_ms=prepare_ms, peak_device_mib=peak_mb, n=N, nnz=g.nnz, k=k, p=p, T=T,
        round_ms=round_ms, round_launches=n_round, round2_ms=ms_r2 / max(n_r2, 1),
        round_q_ms=ms_rq / max(n_rq, 1), alg_bytes=alg, achieved_gbs=achieved,
        selected_count=int(cnt.item()), first_selected=int(idx[0, 0].item()),
    )
    return out, w


def bench_training(args, s2v, torch):
    t0 = time.time()
    w = si.config(5, args.scale)
    g = w.graph
    S = w.x.shape[0]
    log(f"[bench] config 5 generated: n={g.n} nnz={g.nnz} S={S} ({time.time() - t0:.1f}s)")
    ctx = s2v.Context()
    graph = upload(s2v, torch, g)
    N, p, T = g.n, w.p, w.T
    ws = torch.empty(ctx.s2v_workspace_bytes(graph, p, T, S, 1, True), dtype=torch.uint8, device="cuda")
    ctx.s2v_graph_prepare(graph, ws)
    x = torch.from_numpy(w.x).cuda()
    saved = torch.empty((T, N, S, p), device="cuda")
    gsum = torch.empty((S, 1, p), device="cuda")
    action = torch.from_numpy(w.action).cuda()
    target = torch.from_numpy(w.target).cuda()
    loss = torch.empty((1,), device="cuda")
    qp = torch.empty((S,), device="cuda")
    theta0 = s2v.Params.from_numpy(w.theta)
    prm = s2v.Params.from_numpy(w.theta)
    grads = s2v.Params.zeros_like(prm)

    def step():
        # every step starts from the same parameters, then takes w.iters SGD iterations (Sec. 4.5.2)
        for k_ in si.THETA_NAMES:
            prm.t[k_].copy_(theta0.t[k_])
        for _ in range(w.iters):
            # forward + backward in one call (bit for bit the results of s2v_embed_fwd then s2v_embed_bwd)
            ctx.s2v_loss_grad(graph, prm, x, T, S, saved, gsum, action, target, loss, qp, grads, ws)
            ctx.s2v_sgd_step(prm, grads, w.lr)

    steps = max(1, min(args.steps, args.train_steps))
    for _ in range(1):
        step()
    torch.cuda.synchronize()
    ctx.s2v_profile_begin(steps * w.iters * 2 * (T - 1) + 4)
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    (n_f, ms_f), (n_b, ms_b), (n_f2, ms_f2), (n_fl, ms_fl) = ctx.s2v_profile_end()
    alg = round_algorithmic_bytes(N, g.nnz, p, S)
    alg_last = alg - 4 * p * N * S + 8 * N * S      # the last round writes 8-byte mask words, not its rows
    out = dict(ms_per_step=ms, ms_per_iteration=ms / w.iters, steps=steps, iterations=w.iters, S=S, n=N, nnz=g.nnz,
               fwd_round_ms=ms_f / max(n_f, 1), fwd_last_round_ms=ms_fl / max(n_fl, 1),
               bwd_round_ms=ms_b / max(n_b, 1), fwd_round2_ms=ms_f2 / max(n_f2, 1),
               fwd_round_gbs=alg / (ms_f / max(n_f, 1) * 1e-3) / 1e9 if n_f else None,
               fwd_last_round_gbs=alg_last / (ms_fl / max(n_fl, 1) * 1e-3) / 1e9 if n_fl else None,
               fwd_rounds="fwd_round: rounds 3..T-1 (rows walked state by state at this size); fwd_last_round: "
                          "round T, which writes relu-mask words and the graph sums instead of its rows; GB/s = "
                          "algorithmic bytes of the round over its mean duration",
               bwd_rounds="mean over the launched reversed rounds of an iteration, which differ in kind: the first "
                          "gathers 8-byte mask words, the next gathers rows like the forward rounds and also does "
                          "the last reversed round (from the neighbours' scalars) on each tile")
    log(f"[bench] training {ms:.1f} ms/step ({w.iters} iterations); fwd round {out['fwd_round_ms']:.2f} ms, "
        f"last fwd round {out['fwd_last_round_ms']:.2f} ms, "
        f"bwd round {out['bwd_round_ms']:.2f} ms")
    return out


def bench_loop(args, s2v, torch, w4):
    """The rest of the paper's inference step and the whole loop (Alg. 3, Sec. 4.5.1):
    (a) the in-place state update at configuration 4, timed on its own;
    (b) a whole minimum-vertex-cover solve on the paper's largest test-graph shape of Sec. 6.3
        (Erdos-Renyi, 3000 nodes, edge probability 0.15, K = 32, L = 2), one node per evaluation
        versus the adaptive 8/4/2/1 rule.  Random-init parameters: the solution quality means nothing,
        the timing and the evaluation counts do."""
    out = {}
    g = w4.graph
    ctx = s2v.Context()
    graph = upload(s2v, torch, g).mutable_copy()
    N = g.n
    ws = torch.empty(ctx.s2v_workspace_bytes(graph, w4.p, w4.T, 1, 8), dtype=torch.uint8, device="cuda")
    ctx.s2v_graph_prepare(graph, ws)
    x = torch.from_numpy(w4.x[0].copy()).cuda()
    cand = torch.empty(N, dtype=torch.uint8, device="cuda")
    stats = torch.zeros((1, 2), dtype=torch.int32, device="cuda")
    ctx.s2v_residual_update(graph, x, None, None, 0, cand, stats, ws)   # first call removes the covered edges
    torch.cuda.synchronize()
    reps = 10
    t0 = time.perf_counter()
    for _ in range(reps):
        ctx.s2v_residual_update(graph, x, None, None, 0, cand, stats, ws)
    torch.cuda.synchronize()
    out["state_update_full_ms_cfg4"] = (time.perf_counter() - t0) * 1e3 / reps
    st = stats.cpu().numpy()
    out["cfg4_candidates"], out["cfg4_live_entries"] = int(st[0, 0]), int(st[0, 1])
    # incremental updates: ten real steps (embed, score, top-8, update); only the updates are timed
    prm = s2v.Params.from_numpy(w4.theta)
    mu = torch.empty((N, 1, w4.p), device="cuda")
    gsum = torch.empty((1, 1, w4.p), device="cuda")
    q = torch.empty((1, N), device="cuda")
    idx = torch.empty((1, 8), dtype=torch.int32, device="cuda")
    val = torch.empty((1, 8), device="cuda")
    cnt = torch.empty((1,), dtype=torch.int32, device="cuda")
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    t0 = time.perf_counter()
    for a, b in ev:
        ctx.s2v_policy_eval(graph, prm, x.view(1, -1), w4.T, 1, mu, gsum, q, ws)
        ctx.s2v_select_topk(graph, q[0], x, cand, 8, idx, val, cnt, ws)
        a.record()
        ctx.s2v_residual_update(graph, x, idx, cnt, 8, cand, stats, ws)
        b.record()
    torch.cuda.synchronize()
    out["full_step_with_update_ms_cfg4"] = (time.perf_counter() - t0) * 1e3 / reps
    out["state_update_incremental_ms_cfg4"] = sum(a.elapsed_time(b) for a, b in ev) / reps
    del graph, ws, x, cand, mu, q
    torch.cuda.empty_cache()

    n, prob, p, T = 3000, 0.15, 32, 2
    gs = si.erdos_renyi_gnp(n, prob, 777)
    theta = si.thetas(p, 778)
    prm = s2v.Params.from_numpy(theta)
    res = {}
    for adaptive in (False, True):
        graph = upload(s2v, torch, gs).mutable_copy()
        ws = torch.empty(ctx.s2v_workspace_bytes(graph, p, T, 1, 8), dtype=torch.uint8, device="cuda")
        ctx.s2v_graph_prepare(graph, ws)
        x = torch.zeros(n, device="cuda")
        bufs = dict(mu=torch.empty((n, 1, p), device="cuda"), gsum=torch.empty((1, 1, p), device="cuda"),
                    q=torch.empty((1, n), device="cuda"), cand=torch.empty(n, dtype=torch.uint8, device="cuda"),
                    sel_idx=torch.empty((1, 8), dtype=torch.int32, device="cuda"),
                    sel_val=torch.empty((1, 8), device="cuda"), sel_count=torch.empty(1, dtype=torch.int32, device="cuda"),
                    stats=torch.empty((1, 2), dtype=torch.int32, device="cuda"))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        steps, picked, live = ctx.s2v_mvc_inference(graph, prm, x, T, adaptive, 10 * n, bufs["mu"], bufs["gsum"],
                                                    bufs["q"], bufs["cand"], bufs["sel_idx"], bufs["sel_val"],
                                                    bufs["sel_count"], bufs["stats"], ws)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        assert live == 0
        res[adaptive] = dict(seconds=sec, evaluations=steps, cover_size=picked, ms_per_evaluation=sec * 1e3 / steps)
    out["whole_solve_er3000"] = {"graph": f"ER n={n} p={prob} ({gs.nnz // 2} edges), K={p}, L={T}",
                                 "d1": res[False], "adaptive_d": res[True],
                                 "cover_size_ratio": res[True]["cover_size"] / res[False]["cover_size"],
                                 "paper_context_1xV100_s": {"d1": 407.5, "adaptive_d": 109.9, "size_ratio": 1.004}}
    log(f"[bench] state update at cfg 4: full {out['state_update_full_ms_cfg4']:.3f} ms, incremental "
        f"{out['state_update_incremental_ms_cfg4']:.3f} ms, whole step {out['full_step_with_update_ms_cfg4']:.3f} ms; "
        f"whole solve ER(3000,0.15): "
        f"d=1 {res[False]['seconds']:.3f} s / {res[False]['evaluations']} evaluations, "
        f"adaptive {res[True]['seconds']:.3f} s / {res[True]['evaluations']} evaluations")
    return out


def bench_paper_shape(args, s2v, torch):
    """Context line on the paper's own large graph shape (Sec. 6.4: ER, 21 000 nodes, p = 0.15, about
    33 M edges, K = 32, L = 2): one inference step as the paper counts it (embed, score, argmax, state
    update) and one training iteration (forward, loss, backward, SGD) on a 16-state minibatch (the
    paper does not state its batch size).  Next to the paper's 23.8 s / 316.4 s on one V100."""
    t0 = time.time()
    w = si.config(6, args.scale)
    g = w.graph
    N, p, T = g.n, w.p, w.T
    log(f"[bench] paper shape generated: n={N} nnz={g.nnz} ({time.time() - t0:.1f}s)")
    ctx = s2v.Context()
    graph = upload(s2v, torch, g).mutable_copy()
    prm = s2v.Params.from_numpy(w.theta)
    S = 16
    ws = torch.empty(ctx.s2v_workspace_bytes(graph, p, T, S, 8, True), dtype=torch.uint8, device="cuda")
    ctx.s2v_graph_prepare(graph, ws)
    x = torch.zeros(N, device="cuda")
    mu = torch.empty((N, 1, p), device="cuda")
    gsum = torch.empty((1, 1, p), device="cuda")
    q = torch.empty((1, N), device="cuda")
    cand = torch.empty(N, dtype=torch.uint8, device="cuda")
    idx = torch.empty((1, 1), dtype=torch.int32, device="cuda")
    val = torch.empty((1, 1), device="cuda")
    cnt = torch.empty((1,), dtype=torch.int32, device="cuda")
    stats = torch.empty((1, 2), dtype=torch.int32, device="cuda")
    ctx.s2v_residual_update(graph, x, None, None, 0, cand, stats, ws)

    def inf_step():
        ctx.s2v_policy_eval(graph, prm, x.view(1, -1), T, 1, mu, gsum, q, ws)
        ctx.s2v_select_topk(graph, q[0], x, cand, 1, idx, val, cnt, ws)
        ctx.s2v_residual_update(graph, x, idx, cnt, 1, cand, stats, ws)

    for _ in range(3):
        inf_step()
    torch.cuda.synchronize()
    reps = 20
    t0 = time.perf_counter()
    for _ in range(reps):
        inf_step()
    torch.cuda.synchronize()
    inf_ms = (time.perf_counter() - t0) * 1e3 / reps

    # training iteration on the (slightly reduced) graph left by those steps
    xs = torch.from_numpy(si.node_flags(N, 0.05, 99, n_states=S)).cuda()
    xs[:, (x != 0)] = 1.0
    action_np, target_np = si.training_batch(xs.cpu().numpy(), 98)
    action, target = torch.from_numpy(action_np).cuda(), torch.from_numpy(target_np).cuda()
    saved = torch.empty((T, N, S, p), device="cuda")
    gs16 = torch.empty((S, 1, p), device="cuda")
    loss = torch.empty((1,), device="cuda")
    qp = torch.empty((S,), device="cuda")
    grads = s2v.Params.zeros_like(prm)
    theta0 = {k: v.clone() for k, v in prm.t.items()}

    def train_iter():
        ctx.s2v_loss_grad(graph, prm, xs, T, S, saved, gs16, action, target, loss, qp, grads, ws)
        ctx.s2v_sgd_step(prm, grads, 1e-5)

    train_iter()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        train_iter()
    torch.cuda.synchronize()
    train_ms = (time.perf_counter() - t0) * 1e3 / 5
    for k_, v in theta0.items():
        prm.t[k_].copy_(v)
    log(f"[bench] paper shape ER({N}, 0.15): inference step {inf_ms:.3f} ms, training iteration (S={S}) {train_ms:.3f} ms")
    return {"graph": f"ER n={N}, p=0.15 ({g.nnz // 2} edges), K={p}, L={T}",
            "inference_step_ms": inf_ms, "training_iteration_ms_S16": train_ms,
            "paper_1xV100": {"inference_step_s": 23.8, "training_step_s": 316.4}}


def cpu_baseline(w):
    """The float64 oracle, as it stands, on the same inference step (embed + scores + top-k)."""
    import oracle

    oracle.build()
    g = w.graph
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    # whole steps until about ten seconds of CPU work are in (at most four)
    times = []
    while len(times) < 4 and sum(times) < 10e3:
        t0 = time.perf_counter()
        mu = oracle.embed(g.rowptr, g.colidx, g.w, w.theta, w.x[0], w.T)
        _, q = oracle.q_scores(g.graph_off, w.theta, mu)
        oracle.select(g.graph_off, q, w.x[0], None, w.k)
        times.append((time.perf_counter() - t0) * 1e3)
    ms = sum(times) / len(times)
    log(f"[bench] cpu oracle: {ms:.0f} ms per step on {threads} threads ({len(times)} repetitions)")
    return dict(value=ms, unit="ms", cores=threads, kind="oracle",
                sample=f"the whole configuration-4 inference step (n={g.n}, nnz={g.nnz}), mean of {len(times)} "
                       f"repetitions ({sum(times) / 1e3:.1f} s of CPU work)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--train-steps", type=int, default=3)
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the graphs (debugging only; invalid as a result)")
    ap.add_argument("--no-train", action="store_true")
    ap.add_argument("--counters", action="store_true",
                    help="short run for rocprofv3 --pmc: a 1 GiB device copy (calibration) and 3 inference steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-loop", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import torch

    import paper_2105_08764_amd as s2v

    s2v.load_library()  # fails loudly when the HIP library has not been built
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    if args.counters:
        # calibration for byte counters: a plain copy kernel of known size (1 GiB read + 1 GiB written)
        src = torch.empty(1 << 28, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        args.steps, args.warmup, args.no_train, args.no_cpu_baseline = 3, 1, True, True

    ceiling = copy_ceiling_gbs(torch)
    log(f"[bench] streaming ceiling (1 GiB copy, read + write): {ceiling:.0f} GB/s")
    inf, w4 = bench_inference(args, s2v, torch)
    train = None
    if not args.no_train:
        torch.cuda.empty_cache()
        train = bench_training(args, s2v, torch)
    loop = None
    if not args.no_loop and not args.counters:
        torch.cuda.empty_cache()
        loop = bench_loop(args, s2v, torch, w4)
    paper = None
    if not args.no_loop and not args.counters:
        torch.cuda.empty_cache()
        paper = bench_paper_shape(args, s2v, torch)
    cpu = None if args.no_cpu_baseline else cpu_baseline(w4)

    traffic = read_traffic(os.path.join(ROOT, "profiles", "k_round_cfg4_pmc.txt"))
    line = {
        "metric": "ms per RL inference step at 30M edges (embed + Q + top-k)",
        "value": round(inf["ms"], 4),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(inf["ms"], 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "cfg4_er2m: Erdos-Renyi n=2e6, avg degree 30 (60M stored entries), w~U(0.5,1.5), "
                        "x~Bern(0.05), p=64, T=4, top-k with k = 1% of candidates",
            "n_nodes": inf["n"], "nnz": inf["nnz"], "p": inf["p"], "T": inf["T"], "k": inf["k"],
            "scale": args.scale,
        },
        "roofline": {
            "kernel": "k_round<64,false,false,false,false,false,0> (fused CSR gather + theta2 product + relu, rounds 3..T-1; the last round also forms the node term of Eq. 2 and is timed separately)",
            "bound": "hbm",
            "achieved": round(inf["achieved_gbs"], 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(inf["achieved_gbs"] / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "algorithmic_bytes_per_launch": inf["alg_bytes"],
            "avg_launch_ms": round(inf["round_ms"], 4),
            "launches_timed": inf["round_launches"],
            # the same launch on the other byte models: counter-measured traffic, and the compulsory
            # bytes if every embedding row were fetched once (perfect reuse)
            "measured_traffic_gbs": None if traffic is None else round(traffic / (inf["round_ms"] * 1e-3) / 1e9, 1),
            "compulsory_bytes_per_launch": inf["alg_bytes"] - 4 * inf["p"] * (inf["nnz"] - inf["n"]),
            "copy_ceiling_gbs": round(ceiling, 1),
            "frac_of_copy_ceiling": round(inf["achieved_gbs"] / ceiling, 4),
        },
        "cpu_baseline": cpu,
        "round2_from_scalars_ms": round(inf["round2_ms"], 4),
        "last_round_with_q_node_term_ms": round(inf["round_q_ms"], 4),
        "weighted_sum_reading": inf["weighted_sum"],
        "prepare_ms": round(inf["prepare_ms"], 2),
        "peak_device_mib": round(inf["peak_device_mib"], 1),
        "training": train,
        "inference_loop": loop,
        "paper_shape": paper,
        "paper_context": {"inference_step_s_1xV100": 23.8, "training_step_s_1xV100": 316.4,
                          "note": "Summit, ER N=21000 (~33M edges), K=32, L=2; another machine and graph shape"},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
