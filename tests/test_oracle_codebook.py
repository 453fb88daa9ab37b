"""Pins for the oracle's coordinate law and Lloyd-Max codebook (Lemma 1,
eq. (4), Theorem 1).  None of these re-use the oracle's own formulas: they
are closed forms, the paper's printed values, independent quadrature, and
brute force on samples."""
import math

import numpy as np
import pytest
from scipy import integrate

from oracle import turboquant_oracle as o


def _pdf_plain(x, d):
    # Lemma 1 written out directly with math.gamma / lgamma
    logc = math.lgamma(d / 2) - 0.5 * math.log(math.pi) - math.lgamma((d - 1) / 2)
    return math.exp(logc) * (1.0 - x * x) ** ((d - 3) / 2)


@pytest.mark.parametrize("d", [3, 4, 8, 64, 128])
def test_pdf_integrates_to_one_and_has_variance_one_over_d(d):
    m0, _ = integrate.quad(lambda x: float(o.coord_pdf(x, d)), -1, 1, epsabs=1e-13, epsrel=1e-13, limit=400)
    m2, _ = integrate.quad(lambda x: x * x * float(o.coord_pdf(x, d)), -1, 1, epsabs=1e-13, epsrel=1e-13, limit=400)
    assert abs(m0 - 1) < 1e-10
    assert abs(m2 - 1.0 / d) < 1e-10  # a unit vector's squared coordinates sum to 1
    assert abs(float(o.coord_pdf(0.3, d)) - _pdf_plain(0.3, d)) < 1e-12 * _pdf_plain(0.3, d) + 1e-300


@pytest.mark.parametrize("d", [4, 16, 128])
def test_cdf_and_partial_moments_against_quadrature(d):
    s = 1 / math.sqrt(d)
    for lo, hi in [(-1.0, -0.5 * s), (-0.3 * s, 1.1 * s), (0.7 * s, 1.0)]:
        m0, _ = integrate.quad(lambda x: _pdf_plain(x, d), lo, hi, epsabs=1e-14, epsrel=1e-13, limit=400)
        m1, _ = integrate.quad(lambda x: x * _pdf_plain(x, d), lo, hi, epsabs=1e-14, epsrel=1e-13, limit=400)
        m2, _ = integrate.quad(lambda x: x * x * _pdf_plain(x, d), lo, hi, epsabs=1e-14, epsrel=1e-13, limit=400)
        assert abs(float(o.coord_cdf(hi, d) - o.coord_cdf(lo, d)) - m0) < 1e-10
        assert abs(float(o.coord_partial_mean(lo, hi, d)) - m1) < 1e-10
        assert abs(float(o.coord_partial_second_moment(lo, hi, d)) - m2) < 1e-10


def test_coordinate_law_matches_sampled_sphere_points():
    # Lemma 1 against its own statement: coordinates of uniform sphere points
    rng = np.random.default_rng(11)
    d = 6
    g = rng.standard_normal((400000, d))
    x0 = (g / np.linalg.norm(g, axis=1, keepdims=True))[:, 0]
    for t in (-0.6, -0.1, 0.25, 0.7):
        emp = np.mean(x0 <= t)
        assert abs(emp - float(o.coord_cdf(t, d))) < 4 * math.sqrt(0.25 / x0.size)


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_d3_is_the_uniform_quantiser(bits):
    # at d = 3 the exponent (d-3)/2 vanishes: X is uniform on [-1, 1]
    K = 1 << bits
    c, t, cost = o.lloyd_max_codebook(3, bits)
    assert np.allclose(c, -1 + (2 * np.arange(K) + 1) / K, atol=1e-10)
    assert np.allclose(t, -1 + 2 * np.arange(1, K) / K, atol=1e-10)
    assert abs(cost - 1.0 / (3 * K * K)) < 1e-12


@pytest.mark.parametrize("d", [3, 16, 128, 1536, 3072])
def test_b1_closed_form_and_large_d_limit(d, paper):
    c, t, cost = o.lloyd_max_codebook(d, 1)
    e_abs = math.exp(math.lgamma(d / 2) - math.lgamma((d + 1) / 2)) / math.sqrt(math.pi)  # E|X|
    assert abs(c[1] - e_abs) < 1e-12 and abs(c[0] + e_abs) < 1e-12 and t[0] == 0.0
    assert abs(cost - (1.0 / d - e_abs ** 2)) < 1e-13  # D = 1 - d c^2
    if d >= 128:
        # paper: +-sqrt(2/(pi d)) for large d
        assert abs(c[1] * math.sqrt(d) / paper["cent_b1"] - 1) < 2.5e-3


def test_b2_centroids_match_printed_values(paper):
    c, _, _ = o.lloyd_max_codebook(4096, 2)
    s = math.sqrt(4096)
    assert abs(c[2] * s - paper["cent_b2_inner"]) < 5e-4
    assert abs(c[3] * s - paper["cent_b2_outer"]) < 5e-3
    assert np.allclose(c, -c[::-1], atol=0)


@pytest.mark.parametrize("d", [128, 1536, 3072])
def test_dmse_matches_theorem_1_values_and_bounds(d, paper):
    tol = {1: 0.005, 2: 0.0015, 3: 0.005, 4: 0.0006}  # the printed precision
    for b in (1, 2, 3, 4):
        _, _, cost = o.lloyd_max_codebook(d, b)
        D = d * cost  # proof of Theorem 1: D_mse = d C(f_X, b)
        assert abs(D - paper[f"dmse_b{b}"]) < tol[b]
        assert D <= paper["mse_bound_const"] * 4.0 ** -b
        assert D >= 4.0 ** -b  # Theorem 3
    _, _, c1 = o.lloyd_max_codebook(d, 1)
    assert abs(d * c1 / 0.25 - paper["ratio_b1"]) < 0.01


def test_unrounded_gaussian_limit_values():
    # Lloyd-Max for N(0,1) is a textbook table (Max 1960): 0.3634, 0.1175, 0.03454, 0.009497
    d = 1 << 16
    want = {1: 0.3634, 2: 0.1175, 3: 0.03454, 4: 0.009497}
    for b, w in want.items():
        _, _, cost = o.lloyd_max_codebook(d, b)
        assert abs(d * cost - w) < 2e-4 * max(1.0, w / 0.01) * 0.5 + 5e-5


@pytest.mark.parametrize("bits", [5, 6])
def test_panter_dite_bound_at_higher_rates(bits):
    d = 128
    _, _, cost = o.lloyd_max_codebook(d, bits)
    pd = math.sqrt(3) * math.pi / (2 * d) * 4.0 ** -bits  # Theorem 1 proof, b > 4
    # Panter-Dite is a high-resolution asymptote: the optimum approaches it as b grows
    assert 0.85 * pd < cost < 1.03 * pd


@pytest.mark.parametrize("d,bits", [(8, 2), (128, 3), (1536, 4)])
def test_fixed_point_conditions_by_independent_quadrature(d, bits):
    c, t, cost = o.lloyd_max_codebook(d, bits)
    assert np.all(np.diff(c) > 0) and np.allclose(t, 0.5 * (c[1:] + c[:-1]), atol=0)
    edges = np.concatenate(([-1.0], t, [1.0]))
    tot = 0.0
    psum = 0.0
    for k in range(c.size):
        m0, _ = integrate.quad(lambda x: _pdf_plain(x, d), edges[k], edges[k + 1], epsabs=1e-15, epsrel=1e-12, limit=500)
        m1, _ = integrate.quad(lambda x: x * _pdf_plain(x, d), edges[k], edges[k + 1], epsabs=1e-15, epsrel=1e-12, limit=500)
        e2, _ = integrate.quad(lambda x: (x - c[k]) ** 2 * _pdf_plain(x, d), edges[k], edges[k + 1], epsabs=1e-16, epsrel=1e-12, limit=500)
        if m0 > 1e-12:
            assert abs(m1 / m0 - c[k]) < 1e-8 / math.sqrt(d) + 1e-9  # centroid = conditional mean
        tot += e2
        psum += m0 * c[k] ** 2
    assert abs(tot - cost) < 1e-9 * cost + 1e-13
    assert abs(psum - (1.0 / d - cost)) < 1e-10


@pytest.mark.parametrize("d,bits", [(4, 2), (8, 3)])
def test_brute_force_lloyd_on_samples(d, bits):
    # 1-D k-means on a large sample of a sphere coordinate, written out plainly
    rng = np.random.default_rng(5)
    g = rng.standard_normal((1500000, d))
    xs = np.sort((g / np.linalg.norm(g, axis=1, keepdims=True))[:, 0])
    K = 1 << bits
    c = np.quantile(xs, (np.arange(K) + 0.5) / K)
    csum = np.concatenate(([0.0], np.cumsum(xs)))
    for _ in range(300):
        cut = np.searchsorted(xs, 0.5 * (c[1:] + c[:-1]))
        e = np.concatenate(([0], cut, [xs.size]))
        c = (csum[e[1:]] - csum[e[:-1]]) / np.maximum(1, e[1:] - e[:-1])
    want, _, cost = o.lloyd_max_codebook(d, bits)
    assert np.max(np.abs(c - want)) < 4e-3
    emp_cost = np.mean((xs - want[np.searchsorted(0.5 * (want[1:] + want[:-1]), xs, side="right")]) ** 2)
    assert abs(emp_cost - cost) < 0.01 * cost


def test_bucket_masses_and_entropy(paper):
    c, _, _ = o.lloyd_max_codebook(1536, 4)
    p = o.bucket_masses(c, 1536)
    assert abs(p.sum() - 1) < 1e-12 and np.allclose(p, p[::-1], atol=1e-14)
    H = -np.sum(p * np.log2(p))
    assert abs(H - paper["entropy_b4"]) < 0.05  # printed as "approximately 3.8"
    # masses against a direct sample of N(0, 1/d) pushed through the cells (d is large)
    rng = np.random.default_rng(3)
    s = rng.standard_normal(2000000) / math.sqrt(1536)
    t = 0.5 * (c[1:] + c[:-1])
    emp = np.bincount(np.searchsorted(t, s, side="right"), minlength=16) / s.size
    assert np.max(np.abs(emp - p)) < 2e-3


def test_zero_bits_and_fp32_tables():
    c, t, cost = o.lloyd_max_codebook(64, 0)
    assert c.tolist() == [0.0] and t.size == 0 and abs(cost - 1 / 64) < 1e-15
    c32, t32, _ = o.codebook_fp32(128, 3)
    c64, t64, _ = o.lloyd_max_codebook(128, 3)
    assert c32.dtype == np.float32 and t32.dtype == np.float32
    assert np.array_equal(c32, c64.astype(np.float32)) and np.array_equal(t32, t64.astype(np.float32))
    assert np.array_equal(c32, -c32[::-1]) and t32[3] == 0.0
