"""The policy step under HIP graph capture: the library's calls on a prepared graph allocate nothing, read nothing
back and clear their scratch with kernels, so a caller can record a whole step (embedding rounds, scores,
selection: Alg. 3 lines 5-7) once and replay it.  Every replay is compared with the eager call on the same
state, with eager work and synchronisations between the replays and with the inputs changed in place."""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind", ["small", "chain"])
def test_captured_policy_step_replays_like_the_eager_call(kind):
    import torch

    import paper_2105_08764_amd as s2v

    if kind == "small":
        g, p, T, k = si.erdos_renyi_gnp(1000, 0.01, 41), 32, 3, 1        # the fused tail
    else:
        g, p, T, k = si.barabasi_albert(20_000, 5, 42), 64, 3, 50        # the general rounds and the top-k chain
    theta = si.thetas(p, 43)
    N = g.n
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        ctx = s2v.Context()
        graph = s2v.Graph(torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda(), None, None)
        prm = s2v.Params.from_numpy(theta)
        ws = torch.empty(ctx.s2v_workspace_bytes(graph, p, T, 1, k), dtype=torch.uint8, device="cuda")
        ctx.s2v_graph_prepare(graph, ws)
        x = torch.from_numpy(si.node_flags(N, 0.1, 44)[0]).cuda()
        mu = torch.empty((N, 1, p), device="cuda")
        gsum = torch.empty((1, 1, p), device="cuda")
        q = torch.empty((1, N), device="cuda")
        idx = torch.empty((1, k), dtype=torch.int32, device="cuda")
        val = torch.empty((1, k), device="cuda")
        cnt = torch.empty((1,), dtype=torch.int32, device="cuda")

        def step():
            ctx.s2v_policy_select(graph, prm, x, None, T, k, mu, gsum, q, idx, val, cnt, ws)

        step()                      # (warm-up: nothing in the captured region may run for the first time)
        s.synchronize()
    cap = torch.cuda.CUDAGraph()
    with torch.cuda.graph(cap, stream=s):
        step()
    for rep, density in enumerate((0.1, 0.4, 0.0, 0.8)):
        x.copy_(torch.from_numpy(si.node_flags(N, density, 45 + rep)[0]).cuda())
        with torch.cuda.stream(s):
            step()
            s.synchronize()
        want = [t.clone() for t in (mu, gsum, q, idx, val, cnt)]
        for t in (mu, gsum, q, val):
            t.fill_(float("nan"))
        idx.fill_(-7)
        cnt.fill_(-7)
        torch.cuda.synchronize()
        cap.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("mu", "gsum", "q", "idx", "val", "count"), (mu, gsum, q, idx, val, cnt), want):
            assert torch.equal(a, b), (kind, rep, name)
        assert int(cnt[0]) == min(k, int((x == 0).sum()))
