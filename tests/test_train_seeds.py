"""The stored parameter seeds of the gradient parity cases are what the oracle-only search gives."""
import pytest

from tests import gpu_util as gu
from tests import train_cases as tc


def test_every_case_has_a_seed():
    seeds = tc.stored_seeds()
    assert set(seeds) == {(k, p, T, S) for k in tc.KINDS for (p, T, S) in tc.SHAPES}


@pytest.mark.parametrize("kind,p,T,S", [("er", 64, 4, 3), ("er", 32, 5, 16), ("batch", 32, 3, 32), ("ba", 32, 3, 1)])
def test_stored_seed_is_the_first_clear_one(oracle_mod, kind, p, T, S):
    g, x, action, target = tc.inputs(kind, S)
    _, seed = gu.thetas_clear_of_kinks(oracle_mod, g, p, T, x, action, target, tc.first_seed(p, T), tc.theta_scale(kind))
    assert seed == tc.stored_seeds()[(kind, p, T, S)]


def test_detector_flags_a_draw_next_to_a_jump(oracle_mod):
    # er / p = 64 / T = 4 / S = 16: the first draw (seed 145) sits 2e-7 from a point where one relu switches
    # and the gradient changes by 5e-3; the search has to pass over it and two more.
    kind, p, T, S = "er", 64, 4, 16
    g, x, action, target = tc.inputs(kind, S)
    _, seed = gu.thetas_clear_of_kinks(oracle_mod, g, p, T, x, action, target, tc.first_seed(p, T), tc.theta_scale(kind))
    assert seed == tc.stored_seeds()[(kind, p, T, S)] and seed != tc.first_seed(p, T)


def test_every_sweep_case_has_a_seed():
    from tests import sweep_cases as sc

    assert set(sc.stored_seeds()) == set(range(sc.N_CASES))


@pytest.mark.parametrize("case", [0, 7, 13, 21, 33])
def test_stored_sweep_seed_is_the_first_clear_one(oracle_mod, case):
    from tests import sweep_cases as sc

    c = sc.draw(case)
    x, action, target = sc.training_inputs(c)
    _, seed = sc.screened_theta(oracle_mod, c, x, action, target)
    assert seed == sc.stored_seeds()[case]
