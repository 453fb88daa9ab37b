"""Two instances over a split of the channels (Sec. 4.3: outlier channels at one more
bit): the GPU's single set of block-diagonal d = 128 parameters against the oracle's two
independent instances of dimension d_hi and d - d_hi."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2504_19874_amd as tq
import workloads as W
from oracle import turboquant_oracle as o
from tests import parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda"
D = 128


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def words(t):
    return t.cpu().numpy().view(np.uint32)


def instances(d_hi, bits_lo, prod, seed=300):
    """The oracle's two instances and the library's combined parameters, from the same draws."""
    hi_ch = np.sort(np.random.default_rng(seed).permutation(D)[:d_hi])
    g_hi, g_lo = W.gaussian_matrix(d_hi, seed + 1), W.gaussian_matrix(D - d_hi, seed + 2)
    s_hi = W.sketch_matrix(d_hi, seed + 3) if prod else None
    s_lo = W.sketch_matrix(D - d_hi, seed + 4) if prod else None
    inst = []
    for dd, g, s_, b in ((d_hi, g_hi, s_hi, bits_lo + 1), (D - d_hi, g_lo, s_lo, bits_lo)):
        c32, t32, _ = o.codebook_fp32(dd, b)
        inst.append(dict(Pi=o.rotation_from_gaussian(g), S=s_, c32=c32, t32=t32, d=dd, bits=b))
    p = tq.make_mixed_params(D, hi_ch, bits_lo + 1, bits_lo, g_hi, g_lo, s_hi, s_lo)
    return hi_ch, inst[0], inst[1], p


def unpack_split(p, idx_words, d_hi):
    """(idx_hi [n, d_hi], idx_lo [n, d - d_hi]) from the packed words of the split layout."""
    gs, bh, bl = d_hi // 32, p.bits_mse_hi, p.bits_mse
    w = idx_words[:, : p.idx_words]
    hi = o.unpack_planes(w[:, : gs * bh], bh, d_hi) if bh else np.zeros((w.shape[0], d_hi), dtype=np.int32)
    lo = o.unpack_planes(w[:, gs * bh:], bl, D - d_hi) if bl else np.zeros((w.shape[0], D - d_hi), dtype=np.int32)
    return hi, lo


def keys(n, hi_ch, seed=9, bf16=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, D)).astype(np.float32)
    x[:, hi_ch[:4]] *= 20.0  # outlier channels, as in the key-cache recipe
    if n > 5:
        x[5] = 0.0
    if not bf16:
        return x.astype(np.float64), dev(x)
    bits16 = W.f32_to_bf16_bits(x)
    return o.bf16_bits_to_f64(bits16), torch.from_numpy(bits16.view(np.int16)).view(torch.bfloat16).to(DEV)


@pytest.mark.parametrize("d_hi,bits_lo,prod,n,bf16", [
    (32, 1, True, 3000, True), (64, 1, True, 257, False), (32, 2, True, 40000, True), (96, 2, False, 130, False),
    (32, 0, True, 65, False), (64, 3, False, 1000, True),
    # large bf16 batches: the kernel on the bf16 matrix cores (up to 2 + 3 bits), ragged tails
    (64, 1, True, 33000, True), (96, 2, False, 32773, True), (32, 0, True, 34000, True), (64, 3, True, 33000, True),
])
def test_quantize_split(d_hi, bits_lo, prod, n, bf16):
    hi_ch, ihi, ilo, p = instances(d_hi, bits_lo, prod)
    x_or, x_dev = keys(n, hi_ch, bf16=bf16)
    idx = torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device=DEV)
    norm = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV) if prod else None
    gamma = torch.zeros((n, 2), dtype=torch.float32, device=DEV) if prod else None
    if prod:
        tq.tq_quantize_prod(p, x_dev, idx, qjl, gamma, norm)
    else:
        tq.tq_quantize_mse(p, x_dev, idx, norm)
    got_hi, got_lo = unpack_split(p, words(idx), d_hi)
    hi, lo = o.split_channels(D, hi_ch)
    for part, (ch, inst, got) in enumerate(((hi, ihi, got_hi), (lo, ilo, got_lo))):
        xs = x_or[:, ch]
        xh, nu = o.unit_normalise(xs, True)
        y = o.rotate(xh, inst["Pi"])
        idx_or = o.nearest_centroid(y, inst["t32"])
        if inst["bits"]:
            P.check_indices(got, idx_or, y, inst["t32"])
        P.check_close(norm.cpu().numpy()[:, part], nu, 0.0, "norm", rel=3e-6)
        if prod:
            # downstream of the GPU's own indices (teacher forcing)
            _, gamma_or, u_or = o.residual_and_sketch(xh, got, inst["Pi"], inst["S"], inst["c32"])
            P.check_close(gamma.cpu().numpy()[:, part], gamma_or, 0.0, "gamma", rel=1e-5)
            z = o.unpack_signs(words(qjl), D)
            z_part = z[:, :d_hi] if part == 0 else z[:, d_hi:]
            s_norm = np.linalg.norm(inst["S"].astype(np.float64), axis=1)
            P.check_signs(z_part, u_or, s_norm[None, :] * gamma_or[:, None])


@pytest.mark.parametrize("d_hi,bits_lo,prod", [(32, 2, True), (64, 1, False)])
def test_append_split_equals_the_dense_call(d_hi, bits_lo, prod):
    """tq_append with two instances: rows scattered into a larger cache hold exactly what the dense quantiser
    call (checked against the oracle above) writes for the same vectors, and no other slot is touched."""
    hi_ch, _, _, p = instances(d_hi, bits_lo, prod)
    n, first, step = 37, 11, 3
    rows = first + n * step + 5
    _, x_dev = keys(n, hi_ch, bf16=True)

    def arrays(r, fill):
        idx = torch.full((r, p.idx_words), fill, dtype=torch.int32, device=DEV)
        norm = torch.full((r, 2), float("nan"), dtype=torch.float32, device=DEV)
        qjl = torch.full((r, p.qjl_words), fill, dtype=torch.int32, device=DEV) if prod else None
        gamma = torch.full((r, 2), float("nan"), dtype=torch.float32, device=DEV) if prod else None
        return idx, qjl, gamma, norm

    dense, cache = arrays(n, 0), arrays(rows, -1)
    if prod:
        tq.tq_quantize_prod(p, x_dev, *dense)
    else:
        tq.tq_quantize_mse(p, x_dev, dense[0], dense[3])
    tq.tq_append(p, x_dev, *cache, first, step)
    sel = torch.arange(n, device=DEV) * step + first
    rest = torch.ones(rows, dtype=torch.bool, device=DEV)
    rest[sel] = False
    for name, got, want in zip(("idx", "qjl", "gamma", "norm"), cache, dense):
        if got is None:
            continue
        assert torch.equal(got[sel], want), f"{name}: appended rows differ from the dense call"
        other = got[rest]
        assert bool(torch.isnan(other).all() if other.dtype == torch.float32 else (other == -1).all()), f"{name}: stray write"


def random_codes(p, ihi, ilo, d_hi, n, prod, seed=21):
    """Random codes of both instances, in the oracle's form and packed in the split layout."""
    rng = np.random.default_rng(seed)
    res, packed = [], []
    for inst in (ihi, ilo):
        dd, b = inst["d"], inst["bits"]
        r = dict(idx=rng.integers(0, 1 << b, size=(n, dd)).astype(np.int32),
                 norm=np.exp(rng.normal(0, 1, size=n)).astype(np.float32))
        if prod:
            r["qjl"] = rng.integers(0, 2, size=(n, dd)).astype(bool)
            r["gamma"] = rng.uniform(0.05, 0.6, size=n).astype(np.float32)
        res.append(r)
        packed.append(o.pack_planes(r["idx"], b) if b else np.zeros((n, 0), dtype=np.uint32))
    idx_w = np.concatenate(packed, axis=1)
    assert idx_w.shape[1] == p.idx_words
    norm = np.stack([res[0]["norm"], res[1]["norm"]], axis=1)
    qjl_w = gamma = None
    if prod:
        qjl_w = o.pack_signs(np.concatenate([res[0]["qjl"], res[1]["qjl"]], axis=1))
        gamma = np.stack([res[0]["gamma"], res[1]["gamma"]], axis=1)
    return res, idx_w, qjl_w, gamma, norm


@pytest.mark.parametrize("d_hi,bits_lo,prod,n", [(32, 1, True, 777), (64, 2, True, 130), (96, 1, False, 65), (32, 3, False, 300),
                                                (32, 0, True, 40),
                                                # above 8192 vectors: the kernel on the bf16 matrix cores
                                                (32, 1, True, 9000), (64, 2, True, 8200), (96, 1, False, 8500),
                                                (32, 3, False, 9001), (64, 0, True, 8300), (64, 3, True, 8193)])
def test_dequantize_split(d_hi, bits_lo, prod, n):
    hi_ch, ihi, ilo, p = instances(d_hi, bits_lo, prod)
    res, idx_w, qjl_w, gamma, norm = random_codes(p, ihi, ilo, d_hi, n, prod)
    want = o.dequant_split(D, hi_ch, res[0], res[1], ihi, ilo, prod)
    out = torch.zeros((n, D), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, dev(idx_w.view(np.int32)), dev(qjl_w.view(np.int32)) if prod else None,
                     dev(gamma) if prod else None, dev(norm), out)
    scale = np.zeros((n, D))
    hi, lo = o.split_channels(D, hi_ch)
    scale[:, hi] = norm[:, :1] / math.sqrt(d_hi)
    scale[:, lo] = norm[:, 1:] / math.sqrt(D - d_hi)
    P.check_close(out.cpu().numpy(), want, scale, "dequantized coordinate")


@pytest.mark.parametrize("d_hi,bits_lo,prod,n_groups,qpg,npg,topk", [
    (32, 1, True, 8, 4, 1000, 0), (64, 1, True, 2, 5, 2100, 0), (32, 2, True, 1, 4, 130, 5), (96, 2, False, 2, 3, 300, 0),
    (32, 0, True, 1, 1, 77, 0), (64, 3, False, 1, 9, 1500, 4),
    # more than 32 queries per group (served by the same kernel, a block of four queries at a time)
    (64, 2, True, 2, 70, 900, 3),
])
@pytest.mark.parametrize("own_prep", [True, False])
def test_score_split(d_hi, bits_lo, prod, n_groups, qpg, npg, topk, own_prep):
    """own_prep: the scoring kernel rotates its queries itself (needs the transposed matrices);
    without them a preparation kernel runs first."""
    hi_ch, ihi, ilo, p = instances(d_hi, bits_lo, prod)
    if not own_prep:
        p.c.PiT = 0
    n, nq = n_groups * npg, n_groups * qpg
    res, idx_w, qjl_w, gamma, norm = random_codes(p, ihi, ilo, d_hi, n, prod, seed=5)
    q = W.gaussian_queries(nq, D, 3, unit=False)
    q[:, hi_ch[:4]] *= 10.0  # queries see the outlier channels too
    xt = o.dequant_split(D, hi_ch, res[0], res[1], ihi, ilo, prod)
    want = np.concatenate([o.score(q[g * qpg:(g + 1) * qpg], xt[g * npg:(g + 1) * npg]) for g in range(n_groups)])
    scores = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
    ti = torch.zeros((nq, max(1, topk)), dtype=torch.int32, device=DEV)
    p.reserve(n, nq, topk)
    tq.tq_score(p, dev(q), n_groups, qpg, dev(idx_w.view(np.int32)), dev(qjl_w.view(np.int32)) if prod else None,
                dev(gamma) if prod else None, dev(norm), npg, scores, topk, ti if topk else None, None)
    hi, lo = o.split_channels(D, hi_ch)
    q64 = q.astype(np.float64)
    # natural scale of a pair: sum over the instances of |q part| * stored norm
    qs = np.stack([np.linalg.norm(q64[:, hi], axis=1), np.linalg.norm(q64[:, lo], axis=1)], axis=1)
    scale = np.concatenate([qs[g * qpg:(g + 1) * qpg] @ norm[g * npg:(g + 1) * npg].T for g in range(n_groups)])
    got = scores.cpu().numpy()
    P.check_close(got, want, scale, "score")
    if topk:
        assert np.array_equal(ti.cpu().numpy(), o.topk(got, topk))


def test_split_end_to_end_statistics():
    """quantise + score through the library on isotropic keys: the estimate is unbiased and its
    mean squared error is the sum of the two instances' pi/(2 d_part) * d_part C(f_X, b_mse) *
    ||x_part||^2 ||q_part||^2 (Theorem 2's proof per instance), here for 2.5 bits per channel."""
    d_hi, bits_lo, n, nq = 64, 1, 20000, 32
    hi_ch, ihi, ilo, p = instances(d_hi, bits_lo, True)
    rng = np.random.default_rng(31)
    x = rng.standard_normal((n, D)).astype(np.float32)
    q = rng.standard_normal((nq, D)).astype(np.float32)
    idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV)
    gamma = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    norm = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    tq.tq_quantize_prod(p, dev(x), idx, qjl, gamma, norm)
    s = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
    p.reserve(n, nq, 0)
    tq.tq_score(p, dev(q), 1, nq, idx, qjl, gamma, norm, n, s)
    # dequantise agrees with the scores
    xt = torch.zeros((n, D), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, idx, qjl, gamma, norm, xt)
    est = s.cpu().numpy().astype(np.float64)
    x64, q64 = x.astype(np.float64), q.astype(np.float64)
    via = q64 @ xt.cpu().numpy().astype(np.float64).T
    P.check_close(est, via, np.linalg.norm(q64, axis=1)[:, None] * np.linalg.norm(x64, axis=1)[None, :], "score vs <q, x~>")
    exact = q64 @ x64.T
    err = est - exact
    hi, lo = o.split_channels(D, hi_ch)
    var = np.zeros_like(exact)
    for ch, inst in ((hi, ihi), (lo, ilo)):
        cost = o.lloyd_max_codebook(len(ch), inst["bits"])[2]
        var += (math.pi / (2 * len(ch))) * len(ch) * cost * np.sum(q64[:, ch] ** 2, axis=1)[:, None] * \
            np.sum(x64[:, ch] ** 2, axis=1)[None, :]
    assert abs(np.sum(err * exact) / np.sum(exact * exact)) < 0.01
    # the formula is an expectation over S; one fixed 64 x 64 draw sits within ~10 % of it
    assert abs(np.mean(err ** 2) / np.mean(var) - 1) < 0.12


@pytest.mark.parametrize("name", ["C3m", "C3h"])
def test_split_decode_configurations_full_size(name):
    """The 2.5-bit and 3.5-bit decode configurations (Sec. 4.3) at their full size, in the launch shapes
    bench_kernels times: 524288 bf16 keys of 8 heads quantised as two instances (64 + 64 channels with 3 + 2
    resp. 4 + 3 bits), 4 queries per head."""
    cfg = W.CONFIGS[name]
    d_hi, bits_lo = cfg.d_hi, cfg.bits_mse
    hi_ch = W.kv_hi_channels(cfg.n_groups, D, cfg.seed_x, d_hi)
    g_hi, g_lo = W.gaussian_matrix(d_hi, cfg.seed_pi), W.gaussian_matrix(D - d_hi, cfg.seed_pi + 1)
    s_hi, s_lo = W.sketch_matrix(d_hi, cfg.seed_s), W.sketch_matrix(D - d_hi, cfg.seed_s + 1)
    inst = []
    for dd, g, s_, b in ((d_hi, g_hi, s_hi, bits_lo + 1), (D - d_hi, g_lo, s_lo, bits_lo)):
        c32, t32, _ = o.codebook_fp32(dd, b)
        inst.append(dict(Pi=o.rotation_from_gaussian(g), S=s_, c32=c32, t32=t32, d=dd, bits=b))
    ihi, ilo = inst
    p = tq.make_mixed_params(D, hi_ch, bits_lo + 1, bits_lo, g_hi, g_lo, s_hi, s_lo)
    keys = W.kv_keys(cfg.n_groups, cfg.n, D, cfg.seed_x).reshape(-1, D)
    n = keys.shape[0]
    q = W.gaussian_queries(cfg.nq, D, cfg.seed_q, unit=False)
    idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV)
    gamma = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    norm = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    p.reserve(n, cfg.nq, 0)
    tq.tq_quantize_prod(p, torch.from_numpy(keys.view(np.int16)).view(torch.bfloat16).to(DEV), idx, qjl, gamma, norm)
    scores = torch.zeros((cfg.nq, cfg.n), dtype=torch.float32, device=DEV)
    tq.tq_score(p, dev(q), cfg.n_groups, cfg.q_per_group, idx, qjl, gamma, norm, cfg.n, scores)
    got_hi, got_lo = unpack_split(p, words(idx), d_hi)
    z = o.unpack_signs(words(qjl), D)
    g_np, nu_np, s_gpu = gamma.cpu().numpy(), norm.cpu().numpy(), scores.cpu().numpy()
    hi, lo = o.split_channels(D, hi_ch)
    # quantisation against the oracle on a sample of rows from every head
    sample = np.unique(np.concatenate([np.arange(0, 2000), np.arange(n - 2000, n),
                                       np.random.default_rng(5).integers(0, n, size=6000)]))
    x_or = o.bf16_bits_to_f64(keys[sample])
    for part, (ch, it, got) in enumerate(((hi, ihi, got_hi), (lo, ilo, got_lo))):
        xh, nu = o.unit_normalise(x_or[:, ch], True)
        y = o.rotate(xh, it["Pi"])
        P.check_indices(got[sample], o.nearest_centroid(y, it["t32"]), y, it["t32"])
        P.check_close(nu_np[sample, part], nu, 0.0, f"{name} norm", rel=3e-6)
        _, gamma_or, u_or = o.residual_and_sketch(xh, got[sample], it["Pi"], it["S"], it["c32"])
        P.check_close(g_np[sample, part], gamma_or, 0.0, f"{name} gamma", rel=1e-5)
        zp = z[sample][:, :d_hi] if part == 0 else z[sample][:, d_hi:]
        P.check_signs(zp, u_or, np.linalg.norm(it["S"].astype(np.float64), axis=1)[None, :] * gamma_or[:, None])
    # scores of every head against the oracle's estimate from the GPU's own codes
    q64 = q.astype(np.float64)
    qs_n = np.stack([np.linalg.norm(q64[:, hi], axis=1), np.linalg.norm(q64[:, lo], axis=1)], axis=1)
    for g in range(cfg.n_groups):
        rows = slice(g * cfg.n, (g + 1) * cfg.n)
        rh = dict(idx=got_hi[rows], qjl=z[rows][:, :d_hi], gamma=g_np[rows, 0], norm=nu_np[rows, 0])
        rl = dict(idx=got_lo[rows], qjl=z[rows][:, d_hi:], gamma=g_np[rows, 1], norm=nu_np[rows, 1])
        xt = o.dequant_split(D, hi_ch, rh, rl, ihi, ilo, True)
        qsl = slice(g * cfg.q_per_group, (g + 1) * cfg.q_per_group)
        P.check_close(s_gpu[qsl], o.score(q[qsl], xt), qs_n[qsl] @ nu_np[rows].T, f"{name} logits, head {g}")


@pytest.mark.parametrize("d_hi,vbits_lo,kd_hi,n_groups,qpg,npg", [
    (64, 2, 0, 2, 4, 2500),    # the 2.5-bit value cache, ordinary keys (scored inside the read-out kernel)
    (32, 2, 64, 1, 4, 4100),   # keys in two instances as well (scored by tq_score first)
    (96, 1, 0, 1, 5, 700),     # 1 + 2 bits
    (64, 2, 0, 3, 1, 1),       # one token
    (96, 2, 32, 3, 2, 1),      # one token, keys in two instances: the output is one dequantised value vector
])
def test_attend_with_values_in_two_instances(d_hi, vbits_lo, kd_hi, n_groups, qpg, npg):
    """tq_attend with a value cache quantised as two instances (outlier channels one bit wider): softmax of the
    key scores times the oracle's dequantised split values.  Tolerance as in tests/test_gpu_attend.py."""
    v_ch, vhi, vlo, pv = instances(d_hi, vbits_lo, False, seed=500)
    n, nq = n_groups * npg, n_groups * qpg
    vres, v_idx, _, _, v_norm = random_codes(pv, vhi, vlo, d_hi, n, False, seed=31)
    vt = o.dequant_split(D, v_ch, vres[0], vres[1], vhi, vlo, False)
    if kd_hi:
        k_ch, khi, klo, pk = instances(kd_hi, 1, True, seed=600)
        kres, k_idx, k_qjl, k_gamma, k_norm = random_codes(pk, khi, klo, kd_hi, n, True, seed=32)
        k_norm = (k_norm * 0.3).astype(np.float32)
        for r, col in ((kres[0], 0), (kres[1], 1)):
            r["norm"] = k_norm[:, col]
        kt = o.dequant_split(D, k_ch, kres[0], kres[1], khi, klo, True)
        k_dev = (dev(k_idx.view(np.int32)), dev(k_qjl.view(np.int32)), dev(k_gamma), dev(k_norm))
        k_norm_max = float(np.sqrt((k_norm.astype(np.float64) ** 2).sum(axis=1)).max())
    else:
        Pi = o.rotation_from_gaussian(W.gaussian_matrix(D, 700))
        S = W.sketch_matrix(D, 701)
        c32, t32, _ = o.codebook_fp32(D, 2)
        pk = tq.Params(D, 2, torch.from_numpy(Pi), torch.from_numpy(S), c32, t32)
        rng = np.random.default_rng(33)
        idx = rng.integers(0, 4, size=(n, D)).astype(np.int32)
        z = rng.integers(0, 2, size=(n, D)).astype(bool)
        gamma = rng.uniform(0.05, 0.6, size=n).astype(np.float32)
        knorm = np.exp(rng.normal(0, 0.3, size=n)).astype(np.float32)
        kt = o.dequant_prod(idx, z, gamma, Pi, S, c32, knorm)
        k_dev = (dev(o.pack_planes(idx, 2).view(np.int32)), dev(o.pack_signs(z).view(np.int32)), dev(gamma), dev(knorm))
        k_norm_max = float(knorm.max())
    q = W.gaussian_queries(nq, D, 3, unit=False)
    scale = 1.0 / math.sqrt(D)
    out = torch.full((nq, D), float("nan"), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, dev(q), n_groups, qpg, k_dev, (dev(v_idx.view(np.int32)), None, None, dev(v_norm)), npg, scale, out)
    got = out.cpu().numpy().astype(np.float64)
    qn = np.linalg.norm(q.astype(np.float64), axis=1)
    for g in range(n_groups):
        rows, toks = slice(g * qpg, (g + 1) * qpg), slice(g * npg, (g + 1) * npg)
        want = o.attend(q[rows], kt[toks], vt[toks], scale)
        # scale of a dequantised coordinate: |v~| + ||v~|| / sqrt(d) (a coordinate that cancels to nearly zero is still
        # only known to 1e-4 of the vector's typical coordinate), carried through the same softmax
        floor = np.linalg.norm(vt[toks], axis=1, keepdims=True) / math.sqrt(D)
        size = o.attend(q[rows], kt[toks], np.abs(vt[toks]) + floor, scale)
        e = 1e-4 * scale * qn[rows] * k_norm_max
        lim = (P.REL_TOL + np.expm1(2 * e))[:, None] * (size + np.abs(want))
        worst = float((np.abs(got[rows] - want) / np.maximum(lim, 1e-300)).max())
        assert worst <= 1.0, f"attend with split values, group {g}: error {worst:.3f}x the tolerance"


def test_attend_rejects_value_codes_it_does_not_cover():
    """3 + 4 index bits do not fit the kernel's LDS: a clear status, no launch."""
    _, _, _, pv = instances(64, 3, False, seed=510)
    _, _, _, pk = instances(64, 1, True, seed=600)
    with pytest.raises(tq.TurboQuantError, match="UNSUPPORTED|unsupported|outside"):
        z32 = torch.zeros((8, 64), dtype=torch.int32, device=DEV)
        f2 = torch.ones((8, 2), dtype=torch.float32, device=DEV)
        tq.tq_attend(pk, pv, torch.zeros((4, D), device=DEV), 1, 4, (z32, z32, f2, f2), (z32, None, None, f2), 8, 1.0,
                     torch.zeros((4, D), device=DEV))


@pytest.mark.parametrize("d,d_hi,bits_lo,prod,n,nq", [
    (1536, 384, 3, False, 2100, 40),   # the d = 1536 retrieval shape: a quarter of the channels at 4 bits, the rest at 3
    (256, 64, 1, True, 1500, 6),       # few queries, inner-product codes of both instances
    (512, 128, 2, True, 700, 70),
])
def test_split_at_any_dimension_by_two_instances(d, d_hi, bits_lo, prod, n, nq):
    """Sec. 4.3's two instances at a dimension other than 128: the channels of instance hi first, each instance
    an ordinary parameter set of its own dimension that reads its columns of x (and of q) through the row stride
    and writes its columns of the dequantised output the same way; the estimate of <q, x> is the sum of the two
    instances' estimates.  Every call is the library's ordinary one; the oracle's quant_split / dequant_split
    over the same channel split is the reference."""
    hi_ch = np.arange(d_hi)
    dims, bits = (d_hi, d - d_hi), (bits_lo + 1, bits_lo)
    rng = np.random.default_rng(77)
    x = rng.standard_normal((n, d)).astype(np.float32)
    x[:, :8] *= 15.0  # outlier channels lie in instance hi
    x[3] = 0.0
    q = W.gaussian_queries(nq, d, 5, unit=False)
    x_dev, q_dev = dev(x), dev(q)
    xt_dev = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    total = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
    inst, res = [], []
    col = 0
    for part, (dd, b) in enumerate(zip(dims, bits)):
        g = W.gaussian_matrix(dd, 500 + part)
        s_ = W.sketch_matrix(dd, 600 + part) if prod else None
        c32, t32, _ = o.codebook_fp32(dd, b)
        inst.append(dict(Pi=o.rotation_from_gaussian(g), S=s_, c32=c32, t32=t32, d=dd, bits=b))
        p = tq.make_params(dd, b, g, s_).reserve(n, nq, 0)
        xs = x_dev[:, col:col + dd]  # a view: row stride d
        idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
        norm = torch.zeros(n, dtype=torch.float32, device=DEV)
        qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV) if prod else None
        gamma = torch.zeros(n, dtype=torch.float32, device=DEV) if prod else None
        if prod:
            tq.tq_quantize_prod(p, xs, idx, qjl, gamma, norm)
        else:
            tq.tq_quantize_mse(p, xs, idx, norm)
        tq.tq_dequantize(p, idx, qjl, gamma, norm, xt_dev[:, col:col + dd])
        part_scores = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
        tq.tq_score(p, q_dev[:, col:col + dd], 1, nq, idx, qjl, gamma, norm, n, part_scores)
        total += part_scores
        r = dict(idx=o.unpack_planes(words(idx), b, dd), norm=norm.cpu().numpy())
        if prod:
            r["qjl"] = o.unpack_signs(words(qjl), dd)
            r["gamma"] = gamma.cpu().numpy()
        res.append(r)
        col += dd
    # the quantiser of each instance against the oracle's split quantiser
    want_hi, want_lo = o.quant_split(x.astype(np.float64), hi_ch, inst[0], inst[1], prod)
    for r, w, i in zip(res, (want_hi, want_lo), inst):
        P.check_close(r["norm"], w["norm"], 0.0, "norm", rel=3e-6)
        P.check_indices(r["idx"], w["idx"], w["y"], i["t32"])
    # dequantised vectors and scores downstream of the GPU's own codes
    want_xt = o.dequant_split(d, hi_ch, res[0], res[1], inst[0], inst[1], prod)
    scale = np.zeros((n, d))
    scale[:, :d_hi] = res[0]["norm"][:, None] / math.sqrt(d_hi)
    scale[:, d_hi:] = res[1]["norm"][:, None] / math.sqrt(d - d_hi)
    P.check_close(xt_dev.cpu().numpy(), want_xt, scale, "dequantized coordinate")
    bound = sum(np.linalg.norm(q[:, c], axis=1)[:, None] * r["norm"][None, :]
                for c, r in ((slice(0, d_hi), res[0]), (slice(d_hi, d), res[1])))
    P.check_close(total.cpu().numpy(), o.score(q, want_xt), bound, "score")
