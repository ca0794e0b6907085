"""TEST INFRASTRUCTURE ONLY: plain numpy statement of the tuner's generation step.

Follows Sec. 2.3 "GORGO Proxy Design": each weight of the parent is perturbed multiplicatively in log
space by sigma times a standard normal draw and clipped to its range (the unnumbered mutation equation);
an offspring that beats the parent on the objective replaces it, and sigma is steered toward one success
in five proposals (Rechenberg's 1/5 rule).  The paper runs one offspring per step; here a generation has
P candidates, candidate 0 being the unperturbed parent, which reduces to the paper's (1+1) step at P = 2.

The normal draws z are INPUTS (the product draws them with its own counter-based generator and hands the
same numbers to this file in tests), so no random number is generated here.

Parity unpinned by the paper: the 1/5-rule constants (sigma * exp((s - 1/5)/2)) and the parent-selection
fraction mu = max(1, P // 4) are the readings stated here.
"""
import math

import numpy as np


def offspring(theta, sigma, lo, hi, z):
    """params[P,3] from parent theta[3], step size sigma, ranges lo/hi[3] and draws z[P,3] (row 0 unused)."""
    theta = np.asarray(theta, np.float64)
    lo = np.asarray(lo, np.float64)
    hi = np.asarray(hi, np.float64)
    z = np.asarray(z, np.float64)
    P = z.shape[0]
    out = np.empty((P, 3), np.float64)
    out[0] = theta
    for p in range(1, P):
        for k in range(3):
            x = math.exp(math.log(theta[k]) + sigma * z[p, k])
            out[p, k] = min(max(x, lo[k]), hi[k])
    return out


def update(theta, sigma, lo, hi, params, fitness, best_fitness=math.inf, best_theta=None):
    """One generation's update.  fitness[p] is minimised (p95 TTFT in ms).  Returns
    (theta', sigma', best_fitness', best_theta')."""
    params = np.asarray(params, np.float64)
    fitness = np.asarray(fitness, np.float64)
    P = params.shape[0]
    order = sorted(range(P), key=lambda p: (fitness[p], p))       # best first, lowest index on ties
    mu = max(1, P // 4)
    sel = order[:mu]
    if mu == 1:
        new_theta = params[sel[0]].copy()                         # the winner itself replaces the parent
    else:
        new_theta = np.empty(3, np.float64)
        for k in range(3):
            acc = 0.0
            for p in sel:                                         # summed in rank order
                acc += math.log(params[p, k])
            new_theta[k] = math.exp(acc / mu)
    new_theta = np.minimum(np.maximum(new_theta, lo), hi)
    succ = sum(1 for p in range(1, P) if fitness[p] < fitness[0])
    s = succ / (P - 1) if P > 1 else 0.0
    new_sigma = sigma * math.exp((s - 0.2) / 2.0)
    b = order[0]
    if fitness[b] < best_fitness:
        best_fitness, best_theta = float(fitness[b]), params[b].copy()
    return new_theta, new_sigma, best_fitness, best_theta
