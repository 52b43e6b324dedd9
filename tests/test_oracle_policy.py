"""Pins for oracle/policy.py: brute force on tiny vocabularies, closed forms and
the strictness of both policy tests (Sections 3.3 and 3.4)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import policy


def _brute_probs(z):
    e = [math.exp(v) for v in z]
    s = math.fsum(e)
    return [v / s for v in e]


@pytest.mark.parametrize("v", [1, 2, 3, 7, 16])
def test_statistics_against_brute_force(v):
    rng = np.random.default_rng(v)
    for _ in range(20):
        z = rng.normal(0, 3, v)
        p = _brute_probs(list(z))
        assert abs(math.fsum(p) - 1) < 1e-15
        assert np.allclose(policy.softmax(z), p, rtol=1e-13, atol=0)
        assert abs(policy.max_prob(z) - max(p)) < 1e-14
        assert policy.argmax_lowest(z) == max(range(v), key=lambda i: (z[i], -i))
        for t in range(v):
            assert abs(policy.nll(z, t) + math.log(p[t])) < 1e-12
        assert abs(policy.logsumexp(z) - math.log(math.fsum(math.exp(x) for x in z))) < 1e-12


@pytest.mark.parametrize("v", [2, 5, 1024, 250112])
def test_uniform_logits_closed_form(v):
    z = np.full(v, 3.25)
    assert abs(policy.max_prob(z) - 1.0 / v) < 1e-15
    assert abs(policy.nll(z, v - 1) - math.log(v)) < 1e-12
    assert policy.argmax_lowest(z) == 0            # ties resolve to the lowest id


def test_two_point_distribution_exact():
    # logits (ln 3, 0): p = (3/4, 1/4); nll of token 1 is ln 4 (natural log)
    z = np.array([math.log(3.0), 0.0])
    assert abs(policy.max_prob(z) - float(Fraction(3, 4))) < 1e-15
    assert abs(policy.nll(z, 1) - math.log(4.0)) < 1e-15
    assert abs(policy.nll(z, 0) - math.log(4.0 / 3.0)) < 1e-15


def test_stable_for_large_offsets():
    z = np.array([1000.0, 999.0, 998.0])
    assert abs(policy.logsumexp(z) - (1000.0 + math.log(1 + math.exp(-1) + math.exp(-2)))) < 1e-12
    assert abs(policy.logsumexp(z - 2000.0) - (-1000.0 + math.log(1 + math.exp(-1) + math.exp(-2)))) < 1e-12
    assert np.isfinite(policy.nll(z, 2))


def test_shift_invariance_and_scale():
    rng = np.random.default_rng(1)
    z = rng.normal(0, 2, 50)
    assert abs(policy.max_prob(z) - policy.max_prob(z + 7.5)) < 1e-14
    assert abs(policy.nll(z, 3) - policy.nll(z - 11.0, 3)) < 1e-12
    # sharper logits raise the confidence
    assert policy.max_prob(4 * z) > policy.max_prob(z)


def test_top2_gap():
    assert policy.top2_gap(np.array([0.5, 2.0, 1.25, 2.0])) == 0.0
    assert abs(policy.top2_gap(np.array([0.5, 2.0, 1.25])) - 0.75) < 1e-15


def test_fallback_is_strict():
    # two equal logits: max p is exactly 0.5
    z = np.zeros(2)
    assert policy.max_prob(z) == 0.5
    assert not policy.fallback(z, 0.5)          # max p < alpha is false at equality
    assert policy.fallback(z, np.nextafter(0.5, 1.0))
    assert not policy.fallback(z, 0.0)          # alpha_FB = 0 never falls back
    assert policy.fallback(np.array([50.0, 0.0]), 2.0)   # alpha_FB > 1 always falls back


def test_rollback_is_strict():
    z = np.array([0.0, 0.0, 0.0, 0.0])          # nll = ln 4 for every token
    d = policy.nll(z, 2)
    assert not policy.rollback(z, 2, d)         # d > alpha is false at equality
    assert policy.rollback(z, 2, np.nextafter(d, 0.0))
    assert not policy.rollback(z, 2, float("inf"))
    assert policy.rollback(z, 2, -1.0)
