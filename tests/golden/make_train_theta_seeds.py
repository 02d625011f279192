"""Writes tests/golden/train_theta_seeds.txt: for every gradient parity case of
tests/test_gpu_train.py the first parameter seed whose gradient, by the float64 oracle alone, has no
relu jump within float32 rounding of the drawn parameters (tests/gpu_util.thetas_clear_of_kinks says why
that matters and how it is decided).  Calls nothing but the oracle and the input generators.

    python tests/golden/make_train_theta_seeds.py        (about three minutes)
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                       # noqa: E402
from tests import gpu_util as gu    # noqa: E402
from tests import train_cases as tc  # noqa: E402


def main():
    lines = ["# kind p T S seed   (written by tests/golden/make_train_theta_seeds.py; oracle only)"]
    for kind in tc.KINDS:
        for p, T, S in tc.SHAPES:
            g, x, action, target = tc.inputs(kind, S)
            _, seed = gu.thetas_clear_of_kinks(oracle, g, p, T, x, action, target, tc.first_seed(p, T),
                                               tc.theta_scale(kind))
            lines.append(f"{kind} {p} {T} {S} {seed}")
            print(lines[-1], flush=True)
    with open(tc.SEED_FILE, "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
