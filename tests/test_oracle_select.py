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


def test_execute_probability_against_the_two_class_softmax_and_closed_forms():
    # p_0 of Eq. 9 is the class-0 entry of a softmax over the two router outputs; pin the one-argument form against
    # (a) an explicit, max-shifted softmax over (z_e, z_b) pairs written out here, (b) a library softmax, (c) exact
    # rational values sigma(ln(a/b)) = a/(a+b), (d) the symmetry p(z) + p(-z) = 1
    import math
    from fractions import Fraction
    import torch
    rng = np.random.default_rng(9)
    ze = rng.standard_normal(300) * 4.0
    zb = rng.standard_normal(300) * 4.0
    m = np.maximum(ze, zb)
    soft = np.exp(ze - m) / (np.exp(ze - m) + np.exp(zb - m))
    got = orc.execute_probability(ze - zb)
    np.testing.assert_allclose(got, soft, rtol=1e-13)
    lib = torch.softmax(torch.tensor(np.stack([ze, zb], axis=1)), dim=1)[:, 0].numpy()
    np.testing.assert_allclose(got, lib, rtol=1e-13)
    for a, b in [(1, 1), (3, 1), (1, 3), (19, 1), (1, 99), (7, 13)]:
        assert abs(float(orc.execute_probability(math.log(a / b))) - float(Fraction(a, a + b))) < 1e-15
    z = rng.standard_normal(100) * 6.0
    np.testing.assert_allclose(orc.execute_probability(z) + orc.execute_probability(-z), 1.0, rtol=0, atol=1e-15)
    assert float(orc.execute_probability(0.0)) == 0.5


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


# ---- two-output MLP router (Sec. 2.2 / Eq. 9) ------------------------------------------------------------

def _mlp(H, R, seed):
    rng = np.random.default_rng(seed)
    return ((rng.standard_normal((R, H)) * 0.05).astype(np.float32), (rng.standard_normal(R) * 0.1).astype(np.float32),
            (rng.standard_normal((2, R)) * 0.5).astype(np.float32), (rng.standard_normal(2) * 0.1).astype(np.float32))


def test_mlp_router_matches_exact_rational_arithmetic():
    # fp16 activations and fp32 parameters are dyadic rationals: Fraction arithmetic is exact, and the fp64
    # path may differ from it by fp64 rounding only (far below the fp32 rounding of the score)
    from fractions import Fraction
    H, R, T = 12, 5, 7
    W1, b1, W2, b2 = _mlp(H, R, 0)
    x = np.random.default_rng(1).standard_normal((T, H)).astype(np.float16).astype(np.float64)
    z = orc.router_scores_mlp(x, W1, b1, W2, b2)
    for t in range(T):
        u = []
        for r in range(R):
            acc = Fraction(float(b1[r]))
            for k in range(H):
                acc += Fraction(float(W1[r, k])) * Fraction(float(x[t, k]))
            u.append(max(acc, Fraction(0)))
        le = Fraction(float(b2[0])) + sum(Fraction(float(W2[0, r])) * u[r] for r in range(R))
        lb = Fraction(float(b2[1])) + sum(Fraction(float(W2[1, r])) * u[r] for r in range(R))
        exact = float(le - lb)
        assert z[t] == np.float32(exact)                          # the exact value, rounded once to fp32


def test_mlp_router_decision_equals_two_class_softmax():
    H, R, T = 32, 8, 400
    W1, b1, W2, b2 = _mlp(H, R, 2)
    x = np.random.default_rng(3).standard_normal((T, H)).astype(np.float16).astype(np.float64)
    z = orc.router_scores_mlp(x, W1, b1, W2, b2)
    u = np.maximum(x @ W1.astype(np.float64).T + b1, 0)
    logits = u @ W2.astype(np.float64).T + b2
    e = np.exp(logits - logits.max(axis=1, keepdims=True))
    p0 = e[:, 0] / e.sum(axis=1)                                  # Eq. 9 written out
    for theta in (0.5, 0.3, 0.45):
        want = np.nonzero(p0 >= theta)[0]
        got = orc.select_threshold(z, theta)
        near = np.nonzero(np.abs(p0 - theta) < 1e-6)[0]
        assert set(want) - set(near) <= set(got) <= set(want) | set(near)
    assert np.array_equal(orc.select_threshold(z, 0.5), np.nonzero(logits[:, 0] >= logits[:, 1])[0])   # arg-max rule, Eq. 2


def test_mlp_router_with_one_always_active_unit_is_the_linear_router():
    # R = 1, a large positive b1 keeps the ReLU open: z = w2 (w1.x + b1) + b2 is affine in x
    H, T = 16, 50
    rng = np.random.default_rng(4)
    w = (rng.standard_normal(H) * 0.1).astype(np.float32)
    x = rng.standard_normal((T, H)).astype(np.float16).astype(np.float64)
    W1, b1 = w[None, :], np.array([64.0], dtype=np.float32)
    W2, b2 = np.array([[1.0], [0.0]], dtype=np.float32), np.array([-64.0, 0.0], dtype=np.float32)
    z = orc.router_scores_mlp(x, W1, b1, W2, b2)
    lin = orc.router_scores(x, w, 0.0)
    assert np.max(np.abs(z - lin)) <= 64.0 * 2.0 ** -50           # 64 is added and removed in fp64


def test_layer_uses_the_mlp_router_when_given():
    from tests.helpers import TINY, cfg_dict, oracle_layer, to_f64
    import synth_inputs as si
    p, _ = oracle_layer(TINY, 0, 6)
    p.router_mlp = _mlp(TINY.hidden, 4, 5)
    x = to_f64(si.hidden_states(TINY, 20, 6))
    offs, pos = si.equal_sequences(1, 20)
    _, idx, z = orc.layer_forward(x, p, cfg_dict(TINY), offs.numpy(), pos.numpy(), "ratio", 0.5)
    assert np.array_equal(z, orc.router_scores_mlp(x, *p.router_mlp))
    assert np.array_equal(idx, orc.select_ratio(z, 0.5))

