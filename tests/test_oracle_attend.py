"""Pins of the oracle's attention read-out over a quantised key/value cache
(softmax of the Sec. 3.2 scores times the dequantised values): a scalar-loop
brute force and the cases whose answer is known without computing a softmax."""
import math

import numpy as np

from oracle import turboquant_oracle as o


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_attend_matches_scalar_loops():
    q, k, v = _rand(1, 3, 8), _rand(2, 11, 8), _rand(3, 11, 5)
    scale = 0.37
    got = o.attend(q, k, v, scale)
    for a in range(3):
        logit = [scale * sum(q[a, j] * k[i, j] for j in range(8)) for i in range(11)]
        z = sum(math.exp(t) for t in logit)  # no maximum subtracted: small numbers
        for c in range(5):
            want = sum(math.exp(logit[i]) / z * v[i, c] for i in range(11))
            assert abs(got[a, c] - want) < 1e-12


def test_equal_logits_give_the_mean_value():
    q = _rand(4, 2, 16)
    k = np.zeros((40, 16))  # every score is 0
    v = _rand(5, 40, 16)
    np.testing.assert_allclose(o.attend(q, k, v, 1.0), np.broadcast_to(v.mean(axis=0), (2, 16)), atol=1e-13)
    # scale 0 has the same effect whatever the keys are
    np.testing.assert_allclose(o.attend(q, _rand(6, 40, 16), v, 0.0), np.broadcast_to(v.mean(axis=0), (2, 16)),
                               atol=1e-13)


def test_one_dominant_key_returns_its_value():
    q = _rand(7, 1, 16)
    k = _rand(8, 30, 16) * 0.01
    k[17] = q[0]  # aligned with the query
    v = _rand(9, 30, 16)
    out = o.attend(q, k, v, 50.0)
    np.testing.assert_allclose(out[0], v[17], atol=1e-12)


def test_common_shift_of_the_logits_changes_nothing():
    q, k, v = _rand(10, 4, 12), _rand(11, 25, 12), _rand(12, 25, 12)
    base = o.attend(q[:1], k, v, 0.3)
    shift = 3.0 * q[0] / (q[0] @ q[0])  # adds 3 to every score of query 0
    np.testing.assert_allclose(o.attend(q[:1], k + shift, v, 0.3), base, atol=1e-12)
    # large logits do not overflow
    assert np.all(np.isfinite(o.attend(q, 1e3 * k, v, 1.0)))


def test_single_key_and_linearity_in_the_values():
    q, k = _rand(13, 2, 8), _rand(14, 1, 8)
    v = _rand(15, 1, 8)
    np.testing.assert_allclose(o.attend(q, k, v, 2.0), np.broadcast_to(v, (2, 8)), atol=1e-15)
    k, v1, v2 = _rand(16, 9, 8), _rand(17, 9, 8), _rand(18, 9, 8)
    np.testing.assert_allclose(o.attend(q, k, 2.0 * v1 - v2, 0.5),
                               2.0 * o.attend(q, k, v1, 0.5) - o.attend(q, k, v2, 0.5), atol=1e-13)


def test_rows_of_weights_are_a_probability_vector():
    q, k = _rand(19, 3, 8), _rand(20, 50, 8)
    ones = np.ones((50, 1))
    np.testing.assert_allclose(o.attend(q, k, ones, 0.7), np.ones((3, 1)), atol=1e-14)
    # weights are ordered like the scores
    w = o.attend(q, k, np.eye(50), 0.7)
    s = o.score(q, k)
    for a in range(3):
        assert np.array_equal(np.argsort(w[a]), np.argsort(s[a]))
