"""Randomised GPU parity: many small random traces (branching forests, chains, traces that break chain
consistency), replica counts, slot counts, cache sizes, weights and time scales, every formulation, the online
tuner and the baseline policies, each against the CPU oracle."""
import numpy as np
import pytest

import paper_2602_11688_amd as g
from synth import tracegen as tg
from tests.gpu_helpers import check_population, load
from tests.test_gpu_online import _check as check_online
from tests.test_gpu_policies import _check as check_policy

pytestmark = pytest.mark.gpu


def _setup(seed):
    rng = np.random.default_rng(1000 + seed)
    R = int(rng.choice([1, 2, 3, 5, 8, 16, 31, 32, 33, 64]))
    B = int(rng.choice([1, 2, 3, 8, 16]))
    while R * B > 1024:
        B //= 2
    N = int(rng.integers(60, 700))
    kind = seed % 3
    if kind == 0:
        tr = tg.random_forest(seed, N, roots=int(rng.integers(1, 5)), max_blocks=int(rng.integers(4, 60)),
                              grow=int(rng.integers(1, 9)), gap_ms=int(rng.integers(1, 80)), keep=float(rng.choice([0.0, 0.5, 0.85])))
    elif kind == 1:
        tr = tg.random_small(seed, N, R, n_ids=int(rng.integers(10, 200)), max_blocks=int(rng.integers(2, 12)),
                             consistent=True, gap_ms=int(rng.integers(1, 80)))
    else:
        tr = tg.random_small(seed, N, R, n_ids=int(rng.integers(10, 200)), max_blocks=int(rng.integers(2, 12)),
                             consistent=False, gap_ms=int(rng.integers(1, 80)))
    nmax = int(np.diff(tr.blk_off).max())
    C = int(rng.choice([0, nmax, nmax + 1, 2 * nmax + 3, 10 * nmax]))
    model = g.Model(R, B, C, float(rng.choice([0.0, 0.01, 0.05, 0.5])), float(rng.choice([0.0, 1.0, 20.0])))
    rtt = np.round(rng.uniform(0.0, 300.0, R), 1)
    par = rng.uniform(0.0, 2.0, (4, 3))
    if seed % 5 == 0:
        par[0] = [0.0, 0.0, 0.0]
    if seed % 7 == 0:
        par[1] = [-1.0, 1.0, 0.5]
    scale = rng.choice([0.25, 1.0, 3.0, 10.0], 4)
    return rng, tr, model, rtt, par, scale


@pytest.mark.parametrize("seed", range(36))
def test_random_cases(seed):
    rng, tr, model, rtt, par, scale = _setup(seed)
    check_population(tr, model, rtt, par, scale, label=f"fuzz {seed}")
    # (traces that are not chain-consistent run the variants below on block tables)
    window, hop = int(rng.integers(1, 200)), int(rng.integers(1, 70))
    steps = g.online_steps(tr.N, window, hop)
    theta0 = np.clip(par, 0.05, 2.0)
    check_online(tr, model, rtt, theta0, 2.0 * rng.standard_normal((4, steps, 3)), scale, window, hop, lo=[0.05] * 3,
                 hi=[2.0] * 3, sigma0=float(rng.choice([0.0, 0.5, 3.0])))
    for policy in ("least-request", "session-affinity", "random"):
        check_policy(tr, model, rtt, policy, list(scale[:2]), np.array([seed, seed + 1], np.uint64))
