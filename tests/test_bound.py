"""Theorem 3.1's bound as computed by paper_1810_07354_amd.bound (CPU only)."""
import math

import numpy as np
import pytest

from paper_1810_07354_amd import bound


def test_delta_and_bound_by_hand():
    # c = 1/2, one perturbation of norm 1 at iteration 3: Delta = 2^3, bound = log2(1 + 8)
    assert bound.delta_T([1.0], 0.5, first_iteration=3) == 8.0
    assert math.isclose(bound.iteration_cost_bound([1.0], 0.5, 1.0, first_iteration=3), math.log2(9.0))
    # two perturbations: Delta = 1 * 2^0 + 3 * 2^1 = 7
    assert bound.delta_T([1.0, 3.0], 0.5) == 7.0
    assert bound.iteration_cost_bound([0.0, 0.0], 0.9, 2.0) == 0.0
    assert math.isclose(bound.baseline_iterations(1.0, 2.0 ** -10, 0.5), 10.0)
    with pytest.raises(ValueError):
        bound.delta_T([1.0], 1.0)


def test_bound_grows_with_the_perturbation_and_with_its_recency():
    small = bound.iteration_cost_bound([0.1], 0.9, 1.0, first_iteration=20)
    large = bound.iteration_cost_bound([0.2], 0.9, 1.0, first_iteration=20)
    later = bound.iteration_cost_bound([0.1], 0.9, 1.0, first_iteration=30)
    assert small < large and small < later


def test_adversarial_perturbation_meets_the_bound_on_a_quadratic():
    # one eigen-direction, so assumption (3) holds with equality: pushing the iterate straight
    # away from the optimum costs exactly the bound (up to rounding to whole iterations)
    r = bound.quadratic_program(eigenvalues=(0.1,), step=1.0, x0=[1.0], eps=1e-9, perturb_at=40, delta=[0.5])
    assert math.isclose(r["c"], 0.9)
    assert abs(r["iteration_cost"] - r["bound"]) <= 1.0
    assert r["iteration_cost"] > 30


def test_random_perturbations_stay_below_the_bound_on_the_4d_quadratic():
    rng = np.random.default_rng(0)
    for _ in range(200):
        d = rng.normal(size=4) * 10.0 ** rng.uniform(-6, 0)
        r = bound.quadratic_program(delta=d, perturb_at=int(rng.integers(0, 100)), eps=1e-8)
        assert r["iterations_perturbed"] <= r["baseline_bound"] + r["bound"] + 1.0
    zero = bound.quadratic_program(delta=np.zeros(4))
    assert zero["iteration_cost"] == 0 and zero["bound"] == 0.0


def test_smaller_measured_norm_gives_smaller_bound():
    # the use the library's norm is meant for: partial recovery's ||delta'|| <= ||delta||
    # (Theorem 4.1) turns into a smaller cost bound
    full, partial = 17.7, 12.5
    b_full = bound.iteration_cost_bound([full], 0.95, 100.0, first_iteration=30)
    b_part = bound.iteration_cost_bound([partial], 0.95, 100.0, first_iteration=30)
    assert b_part < b_full
