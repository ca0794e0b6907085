"""CPU-only pins of the tuner-step oracle (Sec. 2.3: log-space mutation, clip to [lo,hi], accept-if-better,
Rechenberg 1/5 rule) against closed forms and the (1+1) special case."""
import math

import numpy as np

from oracle import es_oracle as eo

THETA = [0.5, 1.0, 0.1]            # initial weights and ranges of Sec. 4 (prefill weight pinned to 1)
LO = [0.05, 1.0, 0.05]
HI = [2.0, 1.0, 0.5]


def test_zero_draws_reproduce_parent():
    p = eo.offspring(THETA, 0.5, LO, HI, np.zeros((5, 3)))
    np.testing.assert_allclose(p, np.tile(THETA, (5, 1)), rtol=2e-16)


def test_mutation_is_lognormal_and_clipped():
    z = np.array([[0, 0, 0], [1.0, 0.3, -1.0], [10.0, 0, 10.0], [-10.0, 0, -10.0]])
    p = eo.offspring(THETA, 0.5, LO, HI, z)
    assert p[1, 0] == math.exp(math.log(0.5) + 0.5)                 # inside the range: exp(ln x + sigma z)
    assert p[1, 1] == 1.0                                           # lo = hi pins the prefill weight
    assert abs(p[1, 2] - 0.1 * math.exp(-0.5)) < 1e-16 and p[1, 2] == math.exp(math.log(0.1) - 0.5)
    assert p[2].tolist() == [2.0, 1.0, 0.5]                         # learned weights sit on the upper bounds
    assert p[3].tolist() == [0.05, 1.0, 0.05]                       # the lower bound of the queue weight
    rng = np.random.default_rng(0)
    p = eo.offspring(THETA, 0.5, LO, HI, rng.standard_normal((500, 3)))
    assert (p >= LO).all() and (p <= HI).all()
    inside = (p[1:, 0] > 0.05) & (p[1:, 0] < 2.0)
    assert abs(np.log(p[1:, 0][inside]).mean() - math.log(0.5)) < 0.1


def test_one_plus_one_special_case():
    """P=2 is the paper's step: the offspring replaces the parent iff it strictly beats it; sigma grows
    after a success and shrinks after a failure, balanced at one success in five."""
    params = np.array([THETA, [0.8, 1.0, 0.2]])
    th, sg, bf, bt = eo.update(THETA, 0.5, LO, HI, params, [100.0, 90.0])
    assert th.tolist() == [0.8, 1.0, 0.2] and sg == 0.5 * math.exp(0.4) and bf == 90.0 and bt.tolist() == [0.8, 1.0, 0.2]
    th, sg, bf, bt = eo.update(THETA, 0.5, LO, HI, params, [100.0, 100.0])          # tie: parent stays
    assert th.tolist() == THETA and sg == 0.5 * math.exp(-0.1)
    th, sg, _, _ = eo.update(THETA, 0.5, LO, HI, params, [100.0, 130.0])
    assert th.tolist() == THETA and sg == 0.5 * math.exp(-0.1)
    # equilibrium of the step-size rule: 1 success, 4 failures leave sigma where it was
    s = 0.5
    for f in ([1, 0], [0, 1], [0, 1], [0, 1], [0, 1]):
        _, s, _, _ = eo.update(THETA, s, LO, HI, params, f)
    assert abs(s - 0.5) < 1e-15


def test_population_update_is_geometric_mean_of_best_quarter():
    rng = np.random.default_rng(3)
    P = 16
    params = np.column_stack([rng.uniform(0.05, 2, P), np.ones(P), rng.uniform(0.05, 0.5, P)])
    params[0] = THETA
    fit = rng.uniform(10, 20, P)
    th, sg, bf, bt = eo.update(THETA, 0.5, LO, HI, params, fit)
    best4 = np.argsort(fit, kind="stable")[:4]
    np.testing.assert_allclose(th, np.exp(np.log(params[best4]).mean(axis=0)), rtol=1e-14)
    s = (fit[1:] < fit[0]).sum() / 15
    assert sg == 0.5 * math.exp((s - 0.2) / 2)
    assert bf == fit.min() and bt.tolist() == params[fit.argmin()].tolist()


def test_all_equal_fitness_selects_first_indices():
    P = 8
    params = np.column_stack([np.linspace(0.1, 1.5, P), np.ones(P), np.linspace(0.06, 0.4, P)])
    th, sg, _, _ = eo.update(params[0], 0.3, LO, HI, params, np.full(P, 7.0))
    np.testing.assert_allclose(th, np.exp(np.log(params[:2]).mean(axis=0)), rtol=1e-14)
    assert sg == 0.3 * math.exp(-0.1)


def test_best_so_far_is_kept():
    params = np.array([THETA, [0.8, 1.0, 0.2]])
    _, _, bf, bt = eo.update(THETA, 0.5, LO, HI, params, [100.0, 90.0], best_fitness=50.0, best_theta=np.array([1, 1, 0.3]))
    assert bf == 50.0 and bt.tolist() == [1, 1, 0.3]
