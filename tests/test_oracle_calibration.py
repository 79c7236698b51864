"""Pins for the oracle's threshold calibration (CPU only): the two-phase grid search of Sec. 3.4 with
the average execution ratio as objective."""
import math

import numpy as np
import pytest

import synth_inputs as si
from oracle import qtale_oracle as orc
from tests.helpers import TINY, cfg_dict, oracle_layer, to_f64


def _exhaustive(ratio_of_n, target):
    table = {n: ratio_of_n(n) for n in range(1, 51)}
    return min(table, key=lambda n: (abs(table[n] - target), -n)), table


@pytest.mark.parametrize("target", [0.95, 0.8, 0.66, 0.5, 0.31, 0.05])
def test_two_phase_search_finds_the_exhaustive_optimum_for_monotone_ratios(target):
    # any non-increasing R(theta): the coarse winner brackets the crossing, so coarse + fine points
    # contain the best of all 50 grid values
    rng = np.random.default_rng(int(target * 100))
    for _ in range(20):
        steps = np.sort(rng.random(50))[::-1]                  # R(1) >= R(2) >= ... >= R(50)
        fn = lambda n: float(steps[n - 1])
        n, r, seen = orc.two_phase_search(fn, target)
        want, table = _exhaustive(fn, target)
        assert abs(table[n] - target) == abs(table[want] - target)
        assert r == table[n] and len(seen) <= 18               # 10 coarse + at most 8 fine evaluations
        assert list(seen)[:10] == list(range(5, 51, 5))


def test_uniform_probabilities_give_theta_equal_one_minus_ratio():
    # scores whose execute-probabilities are the midpoints (i + 1/2) / N of a uniform grid:
    # the fraction with p >= theta is 1 - theta (up to 1/N), so a target ratio r calibrates to theta = 1 - r
    N = 20000
    u = (np.arange(N) + 0.5) / N
    z = np.log(u / (1.0 - u)).astype(np.float32).reshape(4, N // 4)
    for target, want in [(0.7, 0.30), (0.55, 0.45), (0.93, 0.07), (0.5, 0.50)]:
        theta, r, _ = orc.calibrate_theta_from_scores(z, target)
        assert theta == np.float32(want)
        assert abs(r - target) <= 2.0 / N


def test_targets_outside_the_reachable_range_pick_the_end_of_the_grid():
    z = np.random.default_rng(0).standard_normal((3, 500)).astype(np.float32)
    theta, _, _ = orc.calibrate_theta_from_scores(z, 1.0)
    assert theta == np.float32(0.01)                            # lowest theta executes most
    theta, r, _ = orc.calibrate_theta_from_scores(z, 0.0)
    assert theta == np.float32(0.50) and abs(r - 0.5) < 0.06    # theta stays in (0, 0.5]: about half still runs


def test_ratio_from_scores_is_the_count_of_eq9_decisions():
    z = np.random.default_rng(1).standard_normal((2, 300)).astype(np.float32) * 1.3
    _, _, seen = orc.calibrate_theta_from_scores(z, 0.6)
    for n, r in seen.items():
        p = orc.execute_probability(z)                          # Eq. 9 in the probability domain
        thr = float(np.float32(n / 100.0))
        near = np.abs(p - thr) < 1e-6                           # logit-domain vs probability-domain rounding
        lo = np.count_nonzero((p >= thr) & ~near)
        assert lo <= round(r * z.size) <= lo + np.count_nonzero(near)


def test_stack_calibration_measures_the_realised_ratio():
    shape = TINY
    L, T = 3, 40
    layers = [oracle_layer(shape, l, 5)[0] for l in range(L)]
    for p in layers:                                            # spread the scores: router weight x 40
        p.router_w = (p.router_w * 40).astype(np.float32)
    x = to_f64(si.hidden_states(shape, T, 5))
    offs, pos = si.ragged_sequences([25, 15])
    theta, r, seen = orc.calibrate_theta(x, layers, cfg_dict(shape), offs.numpy(), pos.numpy(), 0.6)
    # every table entry is the realised ratio of an actual threshold-mode run
    for n in (min(seen), max(seen)):
        _, sel, _ = orc.stack_forward(x, layers, cfg_dict(shape), offs.numpy(), pos.numpy(), "threshold", np.float32(n / 100.0))
        assert seen[n] == sum(len(i) for i in sel) / (L * T)
    vals = [seen[n] for n in sorted(seen)]
    assert all(a >= b - 0.05 for a, b in zip(vals, vals[1:]))   # ratio falls (nearly monotonically) with theta
    assert abs(r - 0.6) == min(abs(v - 0.6) for v in seen.values())
