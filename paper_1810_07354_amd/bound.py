"""The iteration-cost bound of Theorem 3.1 as a small CPU calculator, and the quadratic
program of Fig. 3 that illustrates it.

For an update f that contracts by c per iteration (Section 3, assumptions (3) and (4)),
perturbations delta_0 .. delta_T cost at most

    iota <= log(1 + Delta_T / ||x(0) - x*||) / log(1 / c),   Delta_T = sum_l c^(-l) E||delta_l||

extra iterations.  The norms can come from scar_perturbation_norm / scar_partial_recover:
this is how a measured ||delta'|| turns into the quantity the paper's experiments count.
The paper does not give the matrix of its 4-D quadratic program, so `quadratic_program`
takes any spectrum; only the shape of Fig. 3 (cost grows like the bound, and an adversarial
perturbation meets it) can be reproduced, not its numbers.
"""
import math

import numpy as np


def delta_T(norms, c, first_iteration=0):
    """Delta_T = sum over l of c^(-l) * norms[l - first_iteration]."""
    if not 0.0 < c < 1.0:
        raise ValueError("the contraction factor must lie in (0, 1)")
    return float(sum(n * c ** -(first_iteration + i) for i, n in enumerate(norms)))


def iteration_cost_bound(norms, c, dist0, first_iteration=0):
    """Right-hand side of Theorem 3.1 for perturbation norms at iterations
    first_iteration, first_iteration + 1, ..."""
    if dist0 <= 0:
        raise ValueError("||x(0) - x*|| must be positive")
    return math.log1p(delta_T(norms, c, first_iteration) / dist0) / math.log(1.0 / c)


def baseline_iterations(dist0, eps, c):
    """Iterations the unperturbed sequence needs: log(||x(0) - x*|| / eps) / log(1 / c)."""
    return math.log(dist0 / eps) / math.log(1.0 / c)


def quadratic_program(eigenvalues=(1.0, 0.5, 0.2, 0.1), step=1.0, x0=None, eps=1e-6,
                      perturb_at=50, delta=None, max_iter=100000):
    """Gradient descent on l(x) = 1/2 x' diag(eigenvalues) x (x* = 0) with one perturbation
    `delta` added to the iterate at iteration `perturb_at`.  Returns a dict with the
    contraction factor c = max |1 - step * lambda|, the iterations needed with and without
    the perturbation, their difference (the iteration cost) and the bound of Theorem 3.1."""
    lam = np.asarray(eigenvalues, dtype=np.float64)
    rate = 1.0 - step * lam
    c = float(np.max(np.abs(rate)))
    if not 0.0 < c < 1.0:
        raise ValueError("step size does not give a contraction")
    x0 = np.ones_like(lam) if x0 is None else np.asarray(x0, dtype=np.float64)
    delta = np.zeros_like(lam) if delta is None else np.asarray(delta, dtype=np.float64)

    def run(with_delta):
        y = x0.copy()
        for k in range(max_iter):
            if k > perturb_at and np.linalg.norm(y) < eps:
                return k
            if k <= perturb_at and not with_delta and np.linalg.norm(y) < eps:
                return k
            if with_delta and k == perturb_at:
                y = y + delta
            y = rate * y
        return max_iter

    plain, perturbed = run(False), run(True)
    dist0 = float(np.linalg.norm(x0))
    b = iteration_cost_bound([float(np.linalg.norm(delta))], c, dist0, first_iteration=perturb_at)
    # The theorem measures the cost against the unperturbed sequence's own bound
    # log(dist0 / eps) / log(1 / c); a run whose fast directions die out early needs fewer
    # iterations than that, so the cost against the *observed* unperturbed run can exceed b,
    # but the perturbed run never needs more than baseline + b iterations.
    return {"c": c, "iterations_unperturbed": plain, "iterations_perturbed": perturbed,
            "iteration_cost": perturbed - plain, "bound": b,
            "baseline_bound": baseline_iterations(dist0, eps, c)}
