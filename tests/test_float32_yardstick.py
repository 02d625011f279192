"""How often does plain float32 arithmetic miss the float64 gradient at 1e-4 on the gradient parity cases?

Recorded for every first (unscreened) parameter draw of tests/train_cases.py and for every draw the stored
seed list passes over.  The numbers are the yardstick for the HIP path's own miss rate on the same draws
(tests/test_gpu_train_unscreened.py); they are not asserted individually, since float32 sums on the CPU
depend on the host's vector width and thread count."""
import numpy as np

import synth_inputs as si
from tests import float32_yardstick as fy
from tests import relu_decisions as rd
from tests import train_cases as tc


def test_float32_miss_rate_on_first_and_skipped_draws(oracle_mod):
    stored = tc.stored_seeds()
    first_miss, skipped_miss, n_first, n_skipped = [], [], 0, 0
    for kind in tc.KINDS:
        for (p, T, S) in tc.SHAPES:
            g, x, action, target = tc.inputs(kind, S)
            first = tc.first_seed(p, T)
            for seed in range(first, stored[(kind, p, T, S)], 1000) if stored[(kind, p, T, S)] > first else [first]:
                theta = si.thetas(p, seed, tc.theta_scale(kind))
                _, _, og = oracle_mod.loss_grad(g.rowptr, g.colidx, g.w, g.graph_off, theta, x, T, action, target)
                _, _, yg, on, on_head = fy.loss_grad_float32(g, theta, x, T, action, target, decisions=True)
                err = fy.worst_gradient_error(yg, og)
                is_first = seed == first
                n_first += is_first
                n_skipped += seed != stored[(kind, p, T, S)]
                line = f"{kind} p={p} T={T} S={S} seed={seed}{' (first)' if is_first else ''}: float32 vs oracle {err:.2e}"
                if err > 1e-4:
                    (first_miss if is_first else skipped_miss).append((kind, p, T, S, seed))
                    # a miss must be a relu that float32 cannot decide, and vanish on the branch float32 took
                    outs, info = rd.decided_reference(oracle_mod, g, theta, x, T, action, target, on, on_head)
                    dec = fy.worst_gradient_error(yg, outs[0][2])
                    line += f"; on its own branch {dec:.2e} ({info['flips']} unit(s) at |z|/sum|terms| <= {info['worst_ratio']:.1e})"
                    assert dec <= 1e-4
                print(line, flush=True)
    print(f"float32 misses at 1e-4: {len(first_miss)} of {n_first} first draws, {len(skipped_miss)} of {n_skipped} "
          f"draws the stored seed list passes over: {first_miss + skipped_miss}", flush=True)
    # (measured on the build machine: 0 of 24 and 2 of 17)
    assert len(first_miss) <= 3 and len(skipped_miss) <= 6
