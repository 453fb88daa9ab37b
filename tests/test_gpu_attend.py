"""GPU parity of tq_attend (attention read-out over a quantised key/value cache) against the
oracle: softmax of the Sec. 3.2 scores of the key codes times the dequantised value codes.

Tolerance.  A logit carries the score tolerance: |d logit| <= e := 1e-4 * scale * |q| * max nu_K.
Softmax weights then move by a factor within exp(+-2e), so the output moves by at most
(exp(2e) - 1) * sum_i p_i |v~_i| on top of the 1e-4 of its own arithmetic; per coordinate the natural
size of v~_i is nu_V,i / sqrt(d).
"""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import turboquant_oracle as o
from tests import parity as P

pytestmark = pytest.mark.gpu

tq = pytest.importorskip("paper_2504_19874_amd")

DEV = "cuda"


def dev(a):
    return None if a is None else torch.as_tensor(np.ascontiguousarray(a)).to(DEV)


_cache = {}


def setup(d, bits_mse, prod, seed_pi, seed_s):
    key = (d, bits_mse, prod, seed_pi, seed_s)
    if key not in _cache:
        Pi = o.rotation_from_gaussian(W.gaussian_matrix(d, seed_pi))
        S = W.sketch_matrix(d, seed_s) if prod else None
        c32, t32, _ = o.codebook_fp32(d, bits_mse)
        p = tq.Params(d, bits_mse, torch.from_numpy(Pi), None if S is None else torch.from_numpy(S), c32, t32)
        _cache[key] = (p, Pi, S, c32)
    return _cache[key]


def random_codes(rng, n, d, bits_mse, prod, norm_sigma):
    """Uniformly random codes: (oracle-side arrays, device tensors in the packed layout)."""
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool) if prod else None
    gamma = rng.uniform(0.05, 0.6, size=n).astype(np.float32) if prod else None
    norm = np.exp(rng.normal(0, norm_sigma, size=n)).astype(np.float32)
    packed = (dev(o.pack_planes(idx, bits_mse).view(np.int32)) if bits_mse else None,
              dev(o.pack_signs(z).view(np.int32)) if prod else None, dev(gamma), dev(norm))
    return (idx, z, gamma, norm), packed


def dequant(codes, Pi, S, c32):
    idx, z, gamma, norm = codes
    return o.dequant_mse(idx, Pi, c32, norm) if z is None else o.dequant_prod(idx, z, gamma, Pi, S, c32, norm)


def check_attend(out, want, q, scale, k_norm, v_tilde, p_want, d, n_groups, qpg, npg):
    qn = np.linalg.norm(q.astype(np.float64), axis=1)
    for g in range(n_groups):
        rows = slice(g * qpg, (g + 1) * qpg)
        e = 1e-4 * abs(scale) * qn[rows] * float(k_norm[g * npg:(g + 1) * npg].max())
        vt_g = v_tilde[g * npg:(g + 1) * npg]
        # sum_i p_i (|v~_i| + ||v~_i|| / sqrt(d)) per coordinate: the scale of a dequantised coordinate (a coordinate
        # that cancels to nearly zero is still only known to 1e-4 of the vector's typical coordinate)
        size = p_want[rows] @ (np.abs(vt_g) + np.linalg.norm(vt_g, axis=1, keepdims=True) / math.sqrt(vt_g.shape[1]))
        lim = (P.REL_TOL + np.expm1(2 * e))[:, None] * (size + np.abs(want[rows]))
        err = np.abs(out[rows] - want[rows])
        worst = float((err / np.maximum(lim, 1e-300)).max())
        assert worst <= 1.0, f"attend: error {worst:.3f}x the tolerance (max abs err {err.max():.3e})"


CASES = [
    # d, key bits_mse, key prod, value bits_mse, value prod, groups, queries per group, tokens per group
    (128, 2, True, 2, False, 2, 4, 3000),
    (128, 2, True, 1, True, 1, 5, 1100),
    (128, 3, True, 3, False, 3, 1, 700),
    (128, 1, False, 4, False, 1, 4, 2049),
    (128, 2, True, 0, True, 1, 2, 300),
    (64, 2, True, 2, True, 2, 3, 1500),
    (256, 3, False, 2, False, 1, 4, 1025),
    (128, 2, True, 2, False, 1, 4, 1),
    (128, 2, True, 2, False, 8, 4, 4100),
    (128, 3, True, 1, False, 2, 7, 2048),
    (128, 0, True, 3, False, 1, 4, 6200),
    (128, 2, True, 2, True, 2, 4, 2500),
    (128, 3, False, 3, True, 1, 4, 900),
]


@pytest.mark.parametrize("d,kb,kprod,vb,vprod,n_groups,qpg,npg", CASES)
def test_attend(d, kb, kprod, vb, vprod, n_groups, qpg, npg):
    run_attend(d, kb, kprod, vb, vprod, n_groups, qpg, npg, True)


@pytest.mark.parametrize("d,kb,kprod,vb,vprod,n_groups,qpg,npg", [c for c in CASES if c[0] == 128][:5])
def test_attend_with_scores_from_a_scoring_call(d, kb, kprod, vb, vprod, n_groups, qpg, npg):
    """Without the transposed key matrices the keys are scored by tq_score's kernels first and the
    read-out kernel takes the logits from memory."""
    run_attend(d, kb, kprod, vb, vprod, n_groups, qpg, npg, False)


def run_attend(d, kb, kprod, vb, vprod, n_groups, qpg, npg, key_transposes):
    pk, Pik, Sk, ck = setup(d, kb, kprod, 100, 200)
    pv, Piv, Sv, cv = setup(d, vb, vprod, 300, 400)
    n, nq = n_groups * npg, n_groups * qpg
    rng = np.random.default_rng(1000 * d + npg)
    k_codes, k_dev = random_codes(rng, n, d, kb, kprod, 0.3)
    v_codes, v_dev = random_codes(rng, n, d, vb, vprod, 1.0)
    q = W.gaussian_queries(nq, d, 3, unit=False)
    scale = 1.0 / math.sqrt(d)
    kt, vt = dequant(k_codes, Pik, Sk, ck), dequant(v_codes, Piv, Sv, cv)
    want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], kt[g * npg:(g + 1) * npg], vt[g * npg:(g + 1) * npg], scale)
                           for g in range(n_groups)])
    p_want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], kt[g * npg:(g + 1) * npg], np.eye(npg), scale)
                             for g in range(n_groups)])
    out = torch.full((nq, d), float("nan"), dtype=torch.float32, device=DEV)
    keep = pk.c.PiT
    if not key_transposes:
        pk.c.PiT = 0
    try:
        tq.tq_attend(pk, pv, dev(q), n_groups, qpg, k_dev, v_dev, npg, scale, out)
    finally:
        pk.c.PiT = keep
    check_attend(out.cpu().numpy().astype(np.float64), want, q, scale, k_codes[3], vt, p_want, d, n_groups, qpg, npg)


def test_attend_at_the_decode_configuration_full_size():
    """The decode configuration (32 query heads on 8 KV heads, 65536 cached tokens per head, keys b = 3 of Alg. 2)
    with a value cache of the same shape, in the launch configuration the timing harness uses; the oracle
    recomputes two of the eight KV heads."""
    cfg = W.CONFIGS["C3"]
    d, n_groups, qpg, npg = cfg.d, cfg.n_groups, cfg.q_per_group, cfg.n
    pk, Pik, Sk, ck = setup(d, cfg.bits_mse, True, 100, 200)
    pv, Piv, Sv, cv = setup(d, 2, False, 300, 400)
    n, nq = n_groups * npg, n_groups * qpg
    rng = np.random.default_rng(77)
    k_codes, k_dev = random_codes(rng, n, d, cfg.bits_mse, True, 0.3)
    v_codes, v_dev = random_codes(rng, n, d, 2, False, 1.0)
    q = W.gaussian_queries(nq, d, cfg.seed_q, unit=False)
    scale = 1.0 / math.sqrt(d)
    out = torch.full((nq, d), float("nan"), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, dev(q), n_groups, qpg, k_dev, v_dev, npg, scale, out)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    for g in (0, 5):
        rows, toks = slice(g * qpg, (g + 1) * qpg), slice(g * npg, (g + 1) * npg)
        kt = dequant(tuple(None if a is None else a[toks] for a in k_codes), Pik, Sk, ck)
        vt = dequant(tuple(None if a is None else a[toks] for a in v_codes), Piv, Sv, cv)
        want = o.attend(q[rows], kt, vt, scale)
        # sum_i p_i |v~_i| without the npg x npg identity: attend with |v~| as the values
        size = o.attend(q[rows], kt, np.abs(vt), scale)
        qn = np.linalg.norm(q[rows].astype(np.float64), axis=1)
        e = 1e-4 * scale * qn * float(k_codes[3][toks].max())
        lim = (P.REL_TOL + np.expm1(2 * e))[:, None] * (size + np.abs(want))
        err = np.abs(got[rows] - want)
        worst = float((err / lim).max())
        assert worst <= 1.0, f"attend, KV head {g}: error {worst:.3f}x the tolerance"


def test_attend_sharp_softmax_and_padded_rows():
    """A scale large enough that a handful of tokens carry the weight; output rows wider than d."""
    d, n_groups, qpg, npg = 128, 2, 4, 2500
    pk, Pik, Sk, ck = setup(d, 2, True, 100, 200)
    pv, Piv, Sv, cv = setup(d, 2, False, 300, 400)
    n, nq = n_groups * npg, n_groups * qpg
    rng = np.random.default_rng(5)
    k_codes, k_dev = random_codes(rng, n, d, 2, True, 0.3)
    v_codes, v_dev = random_codes(rng, n, d, 2, False, 1.0)
    q = W.gaussian_queries(nq, d, 7, unit=True)
    scale = 60.0
    kt, vt = dequant(k_codes, Pik, Sk, ck), dequant(v_codes, Piv, Sv, cv)
    want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], kt[g * npg:(g + 1) * npg], vt[g * npg:(g + 1) * npg], scale)
                           for g in range(n_groups)])
    p_want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], kt[g * npg:(g + 1) * npg], np.eye(npg), scale)
                             for g in range(n_groups)])
    assert p_want.max(axis=1).min() > 0.02  # the case is what it says
    buf = torch.full((nq, d + 32), float("nan"), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, dev(q), n_groups, qpg, k_dev, v_dev, npg, scale, buf[:, :d])
    assert torch.isnan(buf[:, d:]).all()
    check_attend(buf[:, :d].cpu().numpy().astype(np.float64), want, q, scale, k_codes[3], vt, p_want, d, n_groups,
                 qpg, npg)


def test_attend_without_tokens_gives_zero_rows():
    d = 128
    pk, *_ = setup(d, 2, True, 100, 200)
    pv, *_ = setup(d, 2, False, 300, 400)
    out = torch.full((4, d), float("nan"), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, dev(W.gaussian_queries(4, d, 3, unit=False)), 1, 4, (None, None, None, None),
                 (None, None, None, None), 0, 1.0, out)
    assert torch.equal(out, torch.zeros_like(out))


def test_attend_equals_softmax_of_scores_times_dequantized_values():
    """The library against itself: tq_score + torch softmax + tq_dequantize on codes made by tq_quantize_*."""
    d, n_groups, qpg, npg = 128, 2, 4, 1800
    pk, *_ = setup(d, 2, True, 100, 200)
    pv, *_ = setup(d, 3, False, 300, 400)
    n, nq = n_groups * npg, n_groups * qpg
    keys = torch.from_numpy(W.unit_gaussian_rows(n, d, 21)).to(DEV) * 3.0
    vals = torch.from_numpy(W.unit_gaussian_rows(n, d, 22)).to(DEV) * 2.0
    ki = torch.zeros((n, pk.idx_words), dtype=torch.int32, device=DEV)
    kz = torch.zeros((n, pk.qjl_words), dtype=torch.int32, device=DEV)
    kg = torch.zeros(n, dtype=torch.float32, device=DEV)
    kn = torch.zeros(n, dtype=torch.float32, device=DEV)
    pk.reserve(n, nq, 0)
    tq.tq_quantize_prod(pk, keys, ki, kz, kg, kn)
    vi = torch.zeros((n, pv.idx_words), dtype=torch.int32, device=DEV)
    vn = torch.zeros(n, dtype=torch.float32, device=DEV)
    pv.reserve(n, nq, 0)
    tq.tq_quantize_mse(pv, vals, vi, vn)
    q = torch.from_numpy(W.gaussian_queries(nq, d, 23, unit=False)).to(DEV)
    scale = 1.0 / math.sqrt(d)
    s = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
    tq.tq_score(pk, q, n_groups, qpg, ki, kz, kg, kn, npg, s)
    vt = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(pv, vi, None, None, vn, vt)
    p = torch.softmax(s.double() * scale, dim=1)
    want = torch.cat([p[g * qpg:(g + 1) * qpg] @ vt[g * npg:(g + 1) * npg].double() for g in range(n_groups)])
    out = torch.zeros((nq, d), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, q, n_groups, qpg, (ki, kz, kg, kn), (vi, None, None, vn), npg, scale, out)
    size = torch.cat([p[g * qpg:(g + 1) * qpg] @ vt[g * npg:(g + 1) * npg].double().abs() for g in range(n_groups)])
    assert ((out.double() - want).abs() <= 1e-4 * (size + want.abs())).all()


def _empty_cache(p, rows, prod):
    """Code arrays of `rows` token slots filled with a pattern no quantiser call writes."""
    idx = torch.full((rows, p.idx_words), -1, dtype=torch.int32, device=DEV) if p.idx_words else None
    qjl = torch.full((rows, p.qjl_words), -1, dtype=torch.int32, device=DEV) if prod else None
    gamma = torch.full((rows,), float("nan"), dtype=torch.float32, device=DEV) if prod else None
    norm = torch.full((rows,), float("nan"), dtype=torch.float32, device=DEV)
    return idx, qjl, gamma, norm


def _quantize_dense(p, x, prod):
    idx, qjl, gamma, norm = _empty_cache(p, x.shape[0], prod)
    if prod:
        tq.tq_quantize_prod(p, x, idx, qjl, gamma, norm)
    else:
        tq.tq_quantize_mse(p, x, idx, norm)
    return idx, qjl, gamma, norm


@pytest.mark.parametrize("kb,kprod,vb,vprod", [(2, True, 2, False), (3, True, 1, True), (2, False, 4, False)])
def test_cache_growth_append_then_attend(kb, kprod, vb, vprod):
    """A cache laid out [head][capacity] grows the way decoding grows it (Sec. 4.3: tokens are quantised as
    they arrive): a prefill of each head, then one token for every head per step.  The code rows must be
    bit-identical to quantising the same vectors densely, untouched slots must stay untouched, and the
    read-out over the strided cache must match the oracle on the filled part."""
    d, heads, qpg, cap, prefill, steps = 128, 4, 4, 2600, 2100, 3
    pk, Pik, Sk, ck = setup(d, kb, kprod, 100, 200)
    pv, Piv, Sv, cv = setup(d, vb, vprod, 300, 400)
    rng = np.random.default_rng(5)
    filled = prefill + steps
    keys = (rng.standard_normal((heads, filled, d)) * np.exp(rng.normal(0, 0.3, (heads, filled, 1)))).astype(np.float32)
    vals = (rng.standard_normal((heads, filled, d)) * np.exp(rng.normal(0, 1.0, (heads, filled, 1)))).astype(np.float32)
    kc, vc = _empty_cache(pk, heads * cap, kprod), _empty_cache(pv, heads * cap, vprod)
    for h in range(heads):  # prefill: a run of consecutive slots per head
        tq.tq_append(pk, dev(keys[h, :prefill]), *kc, h * cap, 1)
        tq.tq_append(pv, dev(vals[h, :prefill]), *vc, h * cap, 1)
    for t in range(prefill, filled):  # decode: one token for every head
        tq.tq_append(pk, dev(keys[:, t]), *kc, t, cap)
        tq.tq_append(pv, dev(vals[:, t]), *vc, t, cap)
    torch.cuda.synchronize()

    # the codes: equal to a dense quantiser call on the same vectors, and nothing else written
    for p, x, prod, cache in ((pk, keys, kprod, kc), (pv, vals, vprod, vc)):
        # (head by head: the dense call then runs the same small-batch kernel as the appends, so even the stored
        # floats must be bit-identical; one large batch may take another kernel, equal only within tolerance)
        per_head = [_quantize_dense(p, dev(x[h]), prod) for h in range(heads)]
        dense = [None if per_head[0][k] is None else torch.stack([ph[k].reshape(filled, -1) for ph in per_head]) for k in range(4)]
        for name, got, want in zip(("idx", "qjl", "gamma", "norm"), cache, dense):
            if got is None:
                continue
            got = got.reshape(heads, cap, -1)
            assert torch.equal(got[:, :filled], want), f"{name}: appended rows differ"
            rest = got[:, filled:]
            untouched = torch.isnan(rest).all() if rest.dtype == torch.float32 else (rest == -1).all()
            assert bool(untouched), f"{name}: a slot past the filled part was written"

    # the read-out, against the oracle on the codes the cache holds
    def host_codes(p, cache, prod):
        idx, qjl, gamma, norm = [None if t is None else t.reshape(heads, cap, -1)[:, :filled].reshape(heads * filled, -1).cpu().numpy()
                                 for t in cache]
        i = o.unpack_planes(idx.view(np.uint32), p.bits_mse, d) if p.bits_mse else np.zeros((heads * filled, d), np.int32)
        z = o.unpack_signs(qjl.view(np.uint32), d) if prod else None
        return i, z, None if gamma is None else gamma[:, 0], norm[:, 0]

    k_codes, v_codes = host_codes(pk, kc, kprod), host_codes(pv, vc, vprod)
    kt, vt = dequant(k_codes, Pik, Sk, ck), dequant(v_codes, Piv, Sv, cv)
    nq = heads * qpg
    q = W.gaussian_queries(nq, d, 9, unit=False)
    scale = 1.0 / math.sqrt(d)
    sl = lambda a, g: a[g * filled:(g + 1) * filled]
    want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], sl(kt, g), sl(vt, g), scale) for g in range(heads)])
    p_want = np.concatenate([o.attend(q[g * qpg:(g + 1) * qpg], sl(kt, g), np.eye(filled), scale) for g in range(heads)])
    out = torch.full((nq, d), float("nan"), dtype=torch.float32, device=DEV)
    tq.tq_attend(pk, pv, dev(q), heads, qpg, kc, vc, filled, scale, out, group_stride=cap)
    check_attend(out.cpu().numpy().astype(np.float64), want, q, scale, k_codes[3], vt, p_want, d, heads, qpg, filled)


def test_cache_calls_reject_what_they_do_not_cover():
    p64, *_ = setup(64, 2, True, 100, 200)
    x = torch.zeros((4, 64), dtype=torch.float32, device=DEV)
    cache = _empty_cache(p64, 16, True)
    with pytest.raises(tq.TurboQuantError):
        tq.tq_append(p64, x, *cache, 0, 4)  # d != 128
    p, *_ = setup(128, 2, True, 100, 200)
    x = torch.zeros((4, 128), dtype=torch.float32, device=DEV)
    cache = _empty_cache(p, 16, True)
    with pytest.raises(tq.TurboQuantError):
        tq.tq_append(p, x, *cache, -1, 4)
    with pytest.raises(tq.TurboQuantError):
        tq.tq_append(p, x, *cache, 0, 0)
    out = torch.zeros((4, 64), dtype=torch.float32, device=DEV)
    q = torch.zeros((4, 64), dtype=torch.float32, device=DEV)
    with pytest.raises(tq.TurboQuantError):  # strided groups need the d = 128 kernel
        tq.tq_attend(p64, p64, q, 1, 4, cache, cache, 8, 1.0, out, group_stride=16)
    with pytest.raises(tq.TurboQuantError):  # fewer slots than tokens
        tq.tq_attend(p, p, torch.zeros((4, 128), device=DEV), 1, 4, cache, cache, 8, 1.0,
                     torch.zeros((4, 128), device=DEV), group_stride=4)
