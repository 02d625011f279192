"""s2v_select_topk_noalloc (the selection entry point that allocates nothing: its kernels' scratch is a fixed
array inside the library) against s2v_select_topk, through the C interface: identical idx / val / count, bit
for bit, on two calls in a row of which the second has the smaller input, for the argmax, small-k and
radix-select paths; and its size limits."""
import numpy as np
import pytest

import synth_inputs as si
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _scores(n, seed, ties):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal(n).astype(np.float32)
    if ties:
        q = np.round(q * 4) / 4          # many equal scores: the index order decides
    x = (rng.random(n) < 0.2).astype(np.float32)
    return q.astype(np.float32), x


def _both(dev, ctx, n, q, x, cand, k):
    import torch

    idx, val, cnt = dev.select(q, x, cand, k)
    qd, xd = torch.from_numpy(q).cuda(), torch.from_numpy(x).cuda()
    cd = None if cand is None else torch.from_numpy(cand).cuda()
    i2 = torch.full((1, k), -7, dtype=torch.int32, device="cuda")
    v2 = torch.full((1, k), float("nan"), device="cuda")
    c2 = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ctx.s2v_select_topk_noalloc(n, qd, xd, cd, k, i2, v2, c2)
    torch.cuda.synchronize()
    assert np.array_equal(i2.cpu().numpy(), idx), (n, k)
    assert np.array_equal(v2.cpu().numpy(), val), (n, k)
    assert np.array_equal(c2.cpu().numpy(), cnt), (n, k)
    return cnt


@pytest.mark.parametrize("ties", [False, True])
def test_noalloc_selection_equals_workspace_selection(ties):
    import paper_2105_08764_amd as s2v

    ctx = s2v.Context()
    # first a large input, then a smaller one: the second call finds the first call's scratch contents
    for n, ks in ((300_000, (1, 8, 3000, 200_000)), (70_001, (1, 5, 64, 9000)), (5, (1, 3, 9))):
        g = si.edgeless(n)
        dev = gu.Device(g, 32, 1, k_max=max(ks))
        q, x = _scores(n, 11 + n, ties)
        cand = (np.random.default_rng(n).random(n) < 0.5).astype(np.uint8)
        for k in ks:
            for c in (None, cand):
                print(f"case noalloc n={n} k={k} cand={'mask' if c is not None else 'x'} ties={ties}", flush=True)
                _both(dev, ctx, n, q, x, c, k)
        # no candidate at all
        none = np.zeros(n, dtype=np.uint8)
        assert _both(dev, ctx, n, q, x, none, ks[1])[0] == 0
        del dev


def test_noalloc_limits_and_errors():
    import torch

    import paper_2105_08764_amd as s2v

    ctx = s2v.Context()
    n = 1000
    q = torch.zeros(n, device="cuda")
    x = torch.zeros(n, device="cuda")
    idx = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    val = torch.zeros((1, 4), device="cuda")
    cnt = torch.zeros((1,), dtype=torch.int32, device="cuda")

    def status(fn):
        with pytest.raises(s2v.S2VError) as e:
            fn()
        return e.value.status

    assert status(lambda: ctx.s2v_select_topk_noalloc(s2v.S2V_NOALLOC_MAX_NODES + 1, q, x, None, 4, idx, val, cnt)) == s2v.S2V_ERR_TOO_LARGE
    assert status(lambda: ctx.s2v_select_topk_noalloc(n, q, x, None, s2v.S2V_NOALLOC_MAX_K + 1, idx, val, cnt)) == s2v.S2V_ERR_TOO_LARGE
    assert status(lambda: ctx.s2v_select_topk_noalloc(n, q, x, None, 0, idx, val, cnt)) == s2v.S2V_ERR_INVALID_ARG
    assert status(lambda: ctx.s2v_select_topk_noalloc(n, None, x, None, 4, idx, val, cnt)) == s2v.S2V_ERR_INVALID_ARG
    assert status(lambda: ctx.s2v_select_topk_noalloc(n, q, None, None, 4, idx, val, cnt)) == s2v.S2V_ERR_INVALID_ARG
    assert status(lambda: ctx.s2v_select_topk_noalloc(-1, q, x, None, 4, idx, val, cnt)) == s2v.S2V_ERR_INVALID_ARG
    assert "maximum" in s2v.s2v_status_str(s2v.S2V_ERR_TOO_LARGE)
    # the largest supported sizes run (all scores equal: the k lowest indices come out in order)
    nmax, kmax = s2v.S2V_NOALLOC_MAX_NODES, s2v.S2V_NOALLOC_MAX_K
    qm = torch.zeros(nmax, device="cuda")
    xm = torch.zeros(nmax, device="cuda")
    im = torch.empty((1, kmax), dtype=torch.int32, device="cuda")
    vm = torch.empty((1, kmax), device="cuda")
    ctx.s2v_select_topk_noalloc(nmax, qm, xm, None, kmax, im, vm, cnt)
    torch.cuda.synchronize()
    assert int(cnt.item()) == kmax and torch.equal(im[0], torch.arange(kmax, dtype=torch.int32, device="cuda"))
