"""Pins for the oracle's router score and token selection (CPU only).

Eq. 9: execute iff p_0 >= theta with p = softmax(router logits); theta = 0.5 is the arg-max rule of
Eq. 2; lowering theta raises the execution ratio (Sec. 3.4)."""
import math

import numpy as np
import pytest

from oracle import qtale_oracle as orc


def _scores(T, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(T) * 1.28).astype(np.float32)


def test_router_score_is_the_exactly_rounded_dot_product():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((9, 300)).astype(np.float16).astype(np.float64)
    w = (rng.standard_normal(300) * 0.02).astype(np.float32)
    z = orc.router_scores(x, w, 0.25)
    for t in range(9):
        exact = math.fsum([float(x[t, h]) * float(w[h]) for h in range(300)] + [0.25])
        assert z[t] == np.float32(exact)
    assert z.dtype == np.float32


@pytest.mark.parametrize("T", [1, 7, 64, 1000])
def test_ratio_mode_count_order_and_sort_property(T):
    z = _scores(T, T)
    for r in [0.0, 0.1, 0.3, 0.5, 0.6, 0.8, 1.0]:
        idx = orc.select_ratio(z, r)
        k = int(math.floor(float(np.float32(r)) * T + 0.5))
        assert len(idx) == k == orc.executed_count(r, T)
        assert np.all(np.diff(idx) > 0)
        rest = np.setdiff1d(np.arange(T), idx)
        if k and len(rest):
            assert z[idx].min() >= z[rest].max()
        # independent check against a library sort (stable, descending)
        ref = np.sort(np.argsort(-z.astype(np.float64), kind="stable")[:k])
        assert np.array_equal(idx, ref)


def test_ratio_mode_ties_go_to_the_lower_index():
    z = np.array([0.5, 1.0, 0.5, 0.5, -1.0, 0.5], dtype=np.float32)
    assert list(orc.select_ratio(z, 0.5)) == [0, 1, 2]           # k = 3: the 1.0 and the first two 0.5s
    assert list(orc.select_ratio(z, 2 / 6)) == [0, 1]
    assert list(orc.select_ratio(np.zeros(5, np.float32), 0.6)) == [0, 1, 2]


def test_ratio_sets_are_nested():
    z = _scores(257, 4)
    prev = set()
    for r in np.linspace(0, 1, 21):
        cur = set(orc.select_ratio(z, r).tolist())
        assert prev <= cur
        prev = cur
    assert len(prev) == 257


def test_threshold_half_is_argmax_rule():
    # Eq. 2 on explicit two-class logits vs Eq. 9 with theta = 0.5 on their difference
    rng = np.random.default_rng(1)
    ze = rng.standard_normal(500).astype(np.float32)
    zb = rng.standard_normal(500).astype(np.float32)
    ze[:10] = zb[:10]                                            # exact ties execute (>=)
    z = (ze - zb).astype(np.float32)
    idx = orc.select_threshold(z, 0.5)
    assert np.array_equal(idx, np.nonzero(ze >= zb)[0])
    assert orc.theta_to_logit(0.5) == 0.0


def test_threshold_matches_probability_rule_and_is_monotone():
    z = _scores(400, 2)
    p = 1.0 / (1.0 + np.exp(-z.astype(np.float64)))              # softmax over (z, 0), class 0
    prev = None
    for theta in [0.03, 0.05, 0.1, 0.25, 0.4, 0.5, 0.7]:
        idx = orc.select_threshold(z, theta)
        safe = np.abs(p - theta) > 1e-6                          # away from rounding of the logit
        assert np.array_equal(np.isin(np.arange(400), idx)[safe], (p >= theta)[safe])
        if prev is not None:
            assert set(idx.tolist()) <= prev                      # raising theta shrinks the set
        prev = set(idx.tolist())
    np.testing.assert_allclose(orc.execute_probability(z), p)


def test_threshold_edges():
    z = _scores(20, 3)
    assert len(orc.select_threshold(z, 0.0)) == 20
    assert len(orc.select_threshold(z, -1.0)) == 20
    assert len(orc.select_threshold(z, 1.0)) == 0
    with pytest.raises(ValueError):
        orc.select_threshold(z, float("nan"))
    with pytest.raises(ValueError):
        orc.select_ratio(z, 1.5)
    with pytest.raises(ValueError):
        orc.select_ratio(z, float("nan"))


def test_executed_count_rounding():
    assert orc.executed_count(0.5, 64) == 32
    assert orc.executed_count(0.6, 16384) == 9830
    assert [orc.executed_count(r, 64) for r in (1.0, 0.8, 0.6, 0.4)] == [64, 51, 38, 26]
    assert orc.executed_count(0.5, 1) == 1 and orc.executed_count(0.49, 1) == 0
