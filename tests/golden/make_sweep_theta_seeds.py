"""Writes tests/golden/sweep_theta_seeds.txt: for every case of tests/test_gpu_sweep.py the first parameter
seed whose gradient, by the float64 oracle alone, has no relu jump within float32 rounding of the drawn
parameters (tests/gpu_util.thetas_clear_of_kinks).  Calls nothing but the oracle and the input generators.

    python tests/golden/make_sweep_theta_seeds.py        (a few minutes)
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                         # noqa: E402
from tests import sweep_cases as sc   # noqa: E402


def main():
    lines = ["# case seed   (written by tests/golden/make_sweep_theta_seeds.py; oracle only)"]
    for case in range(sc.N_CASES):
        c = sc.draw(case)
        x, action, target = sc.training_inputs(c)
        _, seed = sc.screened_theta(oracle, c, x, action, target)
        lines.append(f"{case} {seed}   # {c['desc']}")
        print(lines[-1], flush=True)
    with open(sc.SEED_FILE, "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
