"""Pins for the oracle's quantise / dequantise / score / pack / top-k steps
(Alg. 1, Alg. 2, Def. 1, Lemma 4, Theorems 1-2).  They use what the paper and
the mathematics fix: distortion values, unbiasedness, exact variance of the
QJL term, brute-force argmin, hand-built bit patterns."""
import math

import numpy as np
import pytest

import workloads as W
from oracle import turboquant_oracle as o


def _haar(d, seed):
    return o.rotation_from_gaussian(W.gaussian_matrix(d, seed))


def test_rotation_is_orthogonal_and_is_the_qr_factor_with_positive_diagonal():
    G = W.gaussian_matrix(48, 9)
    Pi = o.rotation_from_gaussian(G).astype(np.float64)
    assert np.max(np.abs(Pi @ Pi.T - np.eye(48))) < 1e-6
    R = Pi.T @ G  # must be upper triangular with a positive diagonal
    assert np.max(np.abs(np.tril(R, -1))) < 1e-5 and np.all(np.diag(R) > 0)
    x = W.unit_gaussian_rows(5, 48, 1)
    assert np.allclose(np.linalg.norm(o.rotate(x, Pi), axis=1), 1.0, atol=1e-6)


def test_nearest_centroid_is_the_argmin_of_alg1():
    c32, t32, _ = o.codebook_fp32(128, 3)
    rng = np.random.default_rng(0)
    y = (rng.standard_normal((64, 128)) / math.sqrt(128)).astype(np.float32)
    got = o.nearest_centroid(y, t32)
    dist = np.abs(y.astype(np.float64)[:, :, None] - c32.astype(np.float64)[None, None, :])
    brute = np.argmin(dist, axis=2)
    gap = np.sort(dist, axis=2)
    clear = (gap[:, :, 1] - gap[:, :, 0]) > 1e-6  # away from a tie both must agree
    assert np.array_equal(got[clear], brute[clear]) and clear.mean() > 0.999
    # exactly on a boundary -> upper cell; just below -> lower cell
    yb = np.array([t32, np.nextafter(t32, np.float32(-1))], dtype=np.float32)
    assert np.array_equal(o.nearest_centroid(yb, t32), np.array([np.arange(1, 8), np.arange(0, 7)]))


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_empirical_dmse_matches_theorem_1(bits, paper):
    d, n = 128, 3000
    x = W.unit_gaussian_rows(n, d, 20 + bits)
    Pi = _haar(d, 300 + bits)
    c32, t32, cost = o.codebook_fp32(d, bits)
    idx, nu, _ = o.quant_mse(x, Pi, t32, normalise=False)
    xt = o.dequant_mse(idx, Pi, c32)
    D = np.sum((x - xt) ** 2, axis=1)
    se = D.std() / math.sqrt(n)
    assert abs(D.mean() - d * cost) < 5 * se + 1e-4
    tol = {1: 0.005, 2: 0.0015, 3: 0.005, 4: 0.0006}[bits]
    assert abs(D.mean() - paper[f"dmse_b{bits}"]) < tol + 5 * se
    assert 4.0 ** -bits <= D.mean() <= paper["mse_bound_const"] * 4.0 ** -bits


def test_worst_case_input_has_the_same_distortion_as_random_input():
    # data-oblivious: a basis vector, over many rotations, meets d C(f_X, b)
    d, bits, seeds = 32, 2, 600
    c32, t32, cost = o.codebook_fp32(d, bits)
    e1 = np.zeros((1, d))
    e1[0, 0] = 1.0
    D = []
    for s in range(seeds):
        Pi = _haar(d, 1000 + s)
        idx, _, _ = o.quant_mse(e1, Pi, t32, normalise=False)
        D.append(np.sum((e1 - o.dequant_mse(idx, Pi, c32)) ** 2))
    D = np.array(D)
    assert abs(D.mean() - d * cost) < 4 * D.std() / math.sqrt(seeds)


def test_norm_handling_and_zero_vector():
    d = 64
    Pi = _haar(d, 5)
    c32, t32, _ = o.codebook_fp32(d, 2)
    x = W.unit_gaussian_rows(4, d, 3).astype(np.float64)
    x[1] *= 7.5
    x[2] *= 1e-3
    x[3] = 0.0
    idx, nu, y = o.quant_mse(x, Pi, t32)
    assert np.allclose(nu, [1, 7.5, 1e-3, 0], rtol=1e-6)
    idx_u, _, _ = o.quant_mse(x[:3] / np.linalg.norm(x[:3], axis=1, keepdims=True), Pi, t32, normalise=False)
    assert np.array_equal(idx[:3], idx_u)  # scale invariance of the code
    xt = o.dequant_mse(idx, Pi, c32, nu)
    assert np.all(xt[3] == 0) and np.all(y[3] == 0)
    assert np.allclose(np.linalg.norm(xt[1]) / np.linalg.norm(xt[0]), 7.5 * np.linalg.norm(o.dequant_mse(idx[1:2], Pi, c32)) / np.linalg.norm(o.dequant_mse(idx[0:1], Pi, c32)), rtol=1e-6)
    assert np.all(idx[3] == 2)  # y = 0 sits on the middle boundary -> upper cell


def test_bf16_bit_patterns_are_read_exactly():
    v = np.array([1.0, -2.5, 0.15625, 3.0e-5, -0.0], dtype=np.float32)
    bits = W.f32_to_bf16_bits(v)
    back = o.bf16_bits_to_f64(bits)
    assert np.all(np.abs(back - v) <= np.abs(v) * 2.0 ** -8)
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 0.15625
    assert bits[0] == 0x3F80 and bits[1] == 0xC020


def _many_seed_estimates(d, bits_total, seeds, x, q, kind):
    """estimates <q, x~> over independent (Pi, S) draws, batched"""
    rng = np.random.default_rng(77)
    c32, t32, _ = o.codebook_fp32(d, bits_total - 1 if kind == "prod" else bits_total)
    out = np.empty(seeds)
    for s in range(seeds):
        Pi = o.rotation_from_gaussian(rng.standard_normal((d, d)))
        if kind == "prod":
            S = rng.standard_normal((d, d)).astype(np.float32)
            r = o.quant_prod(x[None], Pi, S, c32, t32, normalise=False)
            xt = o.dequant_prod(r["idx"], r["qjl"], r["gamma"], Pi, S, c32)
        else:
            idx, _, _ = o.quant_mse(x[None], Pi, t32, normalise=False)
            xt = o.dequant_mse(idx, Pi, c32)
        out[s] = o.score(q[None], xt)[0, 0]
    return out


@pytest.mark.parametrize("bits", [1, 2, 3])
def test_prod_is_unbiased_and_meets_theorem_2(bits, paper):
    d, seeds = 48, 4000
    rng = np.random.default_rng(4)
    x = rng.standard_normal(d)
    x /= np.linalg.norm(x)
    q = 0.6 * x + 0.8 * np.linalg.svd(np.vstack([x, rng.standard_normal(d)]).T)[0][:, 1] * 1.0
    q /= np.linalg.norm(q)
    true = float(q @ x)
    est = _many_seed_estimates(d, bits, seeds, x, q, "prod")
    se = est.std() / math.sqrt(seeds)
    assert abs(est.mean() - true) < 4 * se  # Theorem 2, first bullet
    Dprod = np.mean((est - true) ** 2)
    _, _, cost_prev = o.lloyd_max_codebook(d, bits - 1)
    # proof of Theorem 2: D_prod <= pi/(2d) ||q||^2 D_mse(b-1); and the bound of the statement
    assert Dprod <= math.pi / (2 * d) * (d * cost_prev) * 1.08
    assert Dprod <= math.sqrt(3) * math.pi ** 2 / d * 4.0 ** -bits
    assert Dprod >= 4.0 ** -bits / d * 0.5
    # printed values 1.57/d, 0.56/d, 0.18/d are the first line of that chain at large d
    assert d * Dprod < paper[f"dprod_b{bits}"] * 1.08


def test_printed_dprod_values_are_pi_over_two_times_dmse(paper):
    # Theorem 2's refined values follow from its proof: D_prod ~ (pi/2d) D_mse(b-1)
    prev = {1: 1.0, 2: paper["dmse_b1"], 3: paper["dmse_b2"], 4: paper["dmse_b3"]}
    for b in (1, 2, 3, 4):
        assert abs(math.pi / 2 * prev[b] - paper[f"dprod_b{b}"]) < 0.006


def test_qjl_alone_is_unbiased_with_the_exact_variance():
    # bits = 1 total: no MSE stage, r = x.  Lemma 4; the exact per-row variance is
    # (pi/2 ||q||^2 - <q, x>^2) / d for unit x
    d, seeds = 32, 6000
    rng = np.random.default_rng(8)
    x = rng.standard_normal(d)
    x /= np.linalg.norm(x)
    q = rng.standard_normal(d)
    est = _many_seed_estimates(d, 1, seeds, x, q, "prod")
    true = float(q @ x)
    assert abs(est.mean() - true) < 4 * est.std() / math.sqrt(seeds)
    var_exact = (math.pi / 2 * (q @ q) - true ** 2) / d
    assert abs(est.var() / var_exact - 1) < 0.08
    assert est.var() <= math.pi / (2 * d) * (q @ q) * 1.05  # Lemma 4, second bullet


def test_prod_conditional_variance_formula_over_sketch_draws():
    # fixed Pi (so fixed r), many S: Var = gamma^2 ((pi/2)||q||^2 - <q, r/gamma>^2) / d
    d, bits_mse, seeds = 40, 2, 5000
    rng = np.random.default_rng(10)
    Pi = _haar(d, 17)
    c32, t32, _ = o.codebook_fp32(d, bits_mse)
    x = W.unit_gaussian_rows(1, d, 6).astype(np.float64)
    q = rng.standard_normal(d)
    idx, _, _ = o.quant_mse(x, Pi, t32, normalise=False)
    est = np.empty(seeds)
    for s in range(seeds):
        S = rng.standard_normal((d, d)).astype(np.float32)
        r, gamma, u = o.residual_and_sketch(x, idx, Pi, S, c32)
        xt = o.dequant_prod(idx, u >= 0, gamma.astype(np.float32), Pi, S, c32)
        est[s] = q @ xt[0]
    g = float(gamma[0])
    pred = g * g * (math.pi / 2 * (q @ q) - (q @ r[0] / g) ** 2) / d
    assert abs(est.mean() - q @ x[0]) < 4 * est.std() / math.sqrt(seeds)
    assert abs(est.var() / pred - 1) < 0.08


def test_mse_quantiser_bias_is_one_minus_dmse(paper):
    # Sec. 3.2: at b = 1 the MSE quantiser shrinks inner products by 2/pi (large d);
    # in general a Lloyd-Max codebook gives E<q, x~> = (1 - D_mse) <q, x>
    d, seeds = 64, 4000
    rng = np.random.default_rng(12)
    x = rng.standard_normal(d)
    x /= np.linalg.norm(x)
    q = x + 0.3 * rng.standard_normal(d)
    true = float(q @ x)
    for bits in (1, 2):
        _, _, cost = o.lloyd_max_codebook(d, bits)
        est = _many_seed_estimates(d, bits, seeds, x, q, "mse")
        assert abs(est.mean() / true - (1 - d * cost)) < 4 * est.std() / math.sqrt(seeds) / true
        if bits == 1:
            assert abs(est.mean() / true - paper["bias_b1"]) < 0.01


def test_residual_norm_and_gamma():
    d, n = 128, 2000
    x = W.unit_gaussian_rows(n, d, 2)
    Pi, S = _haar(d, 100), W.sketch_matrix(d, 200)
    c32, t32, cost = o.codebook_fp32(d, 2)
    r = o.quant_prod(x, Pi, S, c32, t32, normalise=False)
    # proof of Theorem 1: E||r||^2 = d C(f_X, b)
    g2 = r["gamma"].astype(np.float64) ** 2
    assert abs(g2.mean() - d * cost) < 5 * g2.std() / math.sqrt(n)
    # in the rotated basis the residual is y - c[idx]: same norm
    e = r["y"].astype(np.float64) - c32.astype(np.float64)[r["idx"]]
    assert np.allclose(np.linalg.norm(e, axis=1), r["gamma"], rtol=2e-5)
    assert r["qjl"].dtype == bool and abs(r["qjl"].mean() - 0.5) < 0.01


def test_score_equals_the_rotated_space_form():
    d, n, nq = 64, 50, 7
    x = W.unit_gaussian_rows(n, d, 2).astype(np.float64) * np.linspace(0.5, 3, n)[:, None]
    q = W.gaussian_queries(nq, d, 3, unit=False).astype(np.float64)
    Pi, S = _haar(d, 100), W.sketch_matrix(d, 200)
    c32, t32, _ = o.codebook_fp32(d, 3)
    r = o.quant_prod(x, Pi, S, c32, t32)
    s = o.score(q, o.dequant_prod(r["idx"], r["qjl"], r["gamma"], Pi, S, c32, r["norm"]))
    qr = q @ Pi.astype(np.float64).T
    qs = q @ S.astype(np.float64).T
    z = np.where(r["qjl"], 1.0, -1.0)
    alt = (qr @ c32.astype(np.float64)[r["idx"]].T
           + math.sqrt(math.pi / 2) / d * r["gamma"].astype(np.float64)[None, :] * (qs @ z.T)) * r["norm"].astype(np.float64)[None, :]
    assert np.allclose(s, alt, rtol=1e-10, atol=1e-12)
    # and it does estimate <q, x>: error within a few standard deviations of Theorem 2's bound
    err = s - q @ x.T
    bound = math.sqrt(math.pi / (2 * d) * 0.12) * np.linalg.norm(q, axis=1)[:, None] * np.linalg.norm(x, axis=1)[None, :]
    assert np.mean(np.abs(err) < 3 * bound) > 0.97


def test_pack_planes_hand_built_patterns():
    idx = (np.arange(64) % 4)[None, :].astype(np.int32)  # 0,1,2,3,0,1,...
    w = o.pack_planes(idx, 2)
    assert w.shape == (1, 4) and w.dtype == np.uint32
    assert [hex(v) for v in w[0]] == ["0xaaaaaaaa", "0xcccccccc", "0xaaaaaaaa", "0xcccccccc"]
    one = np.zeros((1, 96), dtype=np.int32)
    one[0, 37] = 5  # group 1, lane 5, planes 0 and 2
    w = o.pack_planes(one, 3)
    want = np.zeros(9, dtype=np.uint32)
    want[3 + 0] = 1 << 5
    want[3 + 2] = 1 << 5
    assert np.array_equal(w[0], want)
    s = np.zeros((1, 64), dtype=bool)
    s[0, [0, 31, 32]] = True
    assert [int(v) for v in o.pack_signs(s)[0]] == [0x80000001, 0x1]
    assert o.pack_planes(np.zeros((3, 32), dtype=np.int32), 0).shape == (3, 0)


@pytest.mark.parametrize("bits", [1, 2, 3, 4])
def test_pack_round_trip(bits):
    rng = np.random.default_rng(bits)
    idx = rng.integers(0, 1 << bits, size=(9, 160)).astype(np.int32)
    w = o.pack_planes(idx, bits)
    assert w.shape == (9, 5 * bits)
    assert np.array_equal(o.unpack_planes(w, bits, 160), idx)
    assert int(sum(bin(int(v)).count("1") for v in w.ravel())) == int(sum(bin(int(v)).count("1") for v in idx.ravel()))


def test_topk_brute_force_and_tie_order():
    rng = np.random.default_rng(1)
    s = rng.standard_normal((5, 200))
    s[0, 17] = s[0, 3] = 9.0  # a tie at the top: lower index first
    got = o.topk(s, 10)
    for r in range(5):
        pairs = sorted(((-s[r, i], i) for i in range(200)))[:10]
        assert [i for _, i in pairs] == got[r].tolist()
    assert got[0, 0] == 3 and got[0, 1] == 17


# ---------------------------------------------------------------------------
# Sec. 4.3: two instances over a channel split
# ---------------------------------------------------------------------------


def _split_instances(d, hi_ch, bits_hi, bits_lo, prod, seed=50):
    inst = []
    for k, (dd, b) in enumerate(((len(hi_ch), bits_hi), (d - len(hi_ch), bits_lo))):
        c32, t32, cost = o.codebook_fp32(dd, b)
        inst.append(dict(Pi=o.rotation_from_gaussian(W.gaussian_matrix(dd, seed + k)),
                         S=W.sketch_matrix(dd, seed + 10 + k) if prod else None, c32=c32, t32=t32, cost=cost))
    return inst


def test_split_quantiser_is_two_ordinary_quantisers():
    """Each instance is an ordinary quantiser of its own channels: on isotropic data its share of
    the squared error is ||x_part||^2 * d_part * C(f_X, b_part) (Theorem 1's proof), whatever the
    other part does; nothing leaks between the channel sets."""
    d, n = 128, 4000
    hi_ch = np.sort(np.random.default_rng(1).permutation(d)[:32])
    ihi, ilo = _split_instances(d, hi_ch, 3, 2, False)
    x = np.random.default_rng(2).standard_normal((n, d))
    x[:, hi_ch] *= 5.0  # a common scale per part changes nothing: each part is normalised on its own
    rh, rl = o.quant_split(x, hi_ch, ihi, ilo, False)
    xt = o.dequant_split(d, hi_ch, rh, rl, ihi, ilo, False)
    hi, lo = o.split_channels(d, hi_ch)
    for ch, inst in ((hi, ihi), (lo, ilo)):
        err = np.sum((x[:, ch] - xt[:, ch]) ** 2, axis=1) / np.sum(x[:, ch] ** 2, axis=1)
        assert abs(err.mean() / (len(ch) * inst["cost"]) - 1) < 0.03
    # an untouched part reproduces the single-instance result on those channels alone
    idx, nu, _ = o.quant_mse(x[:, lo], ilo["Pi"], ilo["t32"])
    assert np.array_equal(idx, rl["idx"]) and np.array_equal(nu, rl["norm"])
    assert np.allclose(xt[:, lo], o.dequant_mse(idx, ilo["Pi"], ilo["c32"], nu))


def test_split_inner_product_estimate_is_unbiased_and_adds_the_variances():
    """<q, x~> of the two-instance prod quantiser: unbiased (Theorem 2 per instance), and its
    variance is the sum of the two instances' pi/(2 d_part) * d_part C(f_X, b_mse of the part) * ||x_part||^2 ||q_part||^2
    (the residual of the MSE stage is what the 1-bit sketch estimates)."""
    d, n = 128, 6000
    hi_ch = np.arange(0, 128, 2)  # 64 channels: (64*3 + 64*2)/128 = 2.5 bits per channel
    ihi, ilo = _split_instances(d, hi_ch, 2, 1, True)  # prod b = 3 and b = 2: MSE stages at 2 and 1 bits
    rng = np.random.default_rng(3)
    x = rng.standard_normal((n, d))
    q = rng.standard_normal((40, d))
    rh, rl = o.quant_split(x, hi_ch, ihi, ilo, True)
    est = o.score(q, o.dequant_split(d, hi_ch, rh, rl, ihi, ilo, True))
    exact = q @ x.T
    err = est - exact
    hi, lo = o.split_channels(d, hi_ch)
    var = np.zeros_like(exact)
    for ch, inst in ((hi, ihi), (lo, ilo)):
        cost_prev = inst["cost"]
        var += (math.pi / (2 * len(ch))) * len(ch) * cost_prev * np.sum(q[:, ch] ** 2, axis=1)[:, None] * \
            np.sum(x[:, ch] ** 2, axis=1)[None, :]
    assert abs(np.sum(err * exact) / np.sum(exact * exact)) < 0.01   # slope 1
    # the formula is an expectation over S; one fixed 64 x 64 draw sits within ~10 % of it
    assert abs(np.mean(err ** 2) / np.mean(var) - 1) < 0.12
