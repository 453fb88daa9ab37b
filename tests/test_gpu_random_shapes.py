"""Seeded random valid shapes through the parity checks of the other GPU test files, and the same entry points
with padded rows, less-aligned pointers and guard values around every output.

The fixed parameter lists of the other files pin the tile sizes and thresholds their authors knew about; these
draws cover the combinations nobody listed (a sweep of this kind found a residual norm off by more than its
tolerance at a 4-bit MSE stage with fp32 input, and wrong codes for bf16 rows at d = 128 that were only 8-byte
aligned).  Every case is printed before it runs so that a failure names its shape."""
import math
import random

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2504_19874_amd as tq
import workloads as W
from oracle import turboquant_oracle as o
from tests import parity as P
from tests import test_gpu_attend as TA
from tests import test_gpu_parity as T
from tests import test_gpu_split as TS

pytestmark = pytest.mark.gpu
DEV = "cuda"
GUARD_I, GUARD_F = -1515870811, 12345.0  # 0xA5A5A5A5


def _n_at_128(rnd):
    """Batch sizes around the thresholds at which the d = 128 calls change kernels."""
    return rnd.choice([rnd.randint(1, 600), rnd.randint(8100, 8300), rnd.randint(24400, 24700), rnd.randint(32000, 40000)])


def _draw(rnd):
    kind = rnd.choice(["mse", "prod", "prod", "deq", "score", "score", "attend", "topk", "split_q", "split_d", "big_d"])
    if kind in ("mse", "prod", "deq"):
        d = rnd.choice([128, 128, 128, 32, 64, 96, 160, 256, 384, 512])
        n = _n_at_128(rnd) if d == 128 else rnd.randint(1, 700)
        src = rnd.choice(["unit", "f32", "bf16", "bf16unit"])
        if kind == "mse":
            return T.test_quantize_mse, (d, rnd.randint(1, 4), n, src)
        if kind == "prod":
            return T.test_quantize_prod, (d, rnd.randint(0, 4), n, src)
        prod = rnd.random() < 0.5
        return T.test_dequantize, (d, rnd.randint(0 if prod else 1, 4), n, prod, rnd.random() < 0.5)
    if kind == "score":
        d = rnd.choice([128, 128, 128, 64, 96, 256, 384, 512, 640])
        prod = rnd.random() < 0.5
        g, qpg = rnd.choice([1, 1, 2, 3, 8, 33]), rnd.choice([1, 2, 3, 4, 5, 9, 32, 33, 64, 70, 130])
        npg = rnd.choice([rnd.randint(1, 300), rnd.randint(2040, 2060), rnd.randint(1000, 9000)])
        npg = max(1, min(npg, 6_000_000 // (g * d), 3_000_000 // (g * qpg)))
        topk = rnd.choice([0, 0, 1, 5, 10, 16, 20])
        return T.test_score_and_topk, (d, rnd.randint(0 if prod else 1, 4), prod, g, qpg, npg, topk if topk <= npg else 0)
    if kind == "attend":
        kprod, vprod = rnd.random() < 0.6, rnd.random() < 0.4
        npg = rnd.choice([rnd.randint(1, 300), rnd.randint(2040, 2060), rnd.randint(300, 7000)])
        return TA.test_attend, (rnd.choice([128, 128, 128, 64, 256]), rnd.randint(0 if kprod else 1, 4), kprod,
                                rnd.randint(0 if vprod else 1, 4), vprod, rnd.choice([1, 2, 3, 8]),
                                rnd.choice([1, 2, 4, 5, 7, 8, 33]), npg)
    if kind == "topk":
        prod = rnd.random() < 0.5
        g, qpg = rnd.choice([1, 1, 2, 3]), rnd.choice([33, 65, 100, 129, 257, 300])
        npg = rnd.choice([rnd.randint(1, 50), rnd.randint(200, 3000), rnd.randint(3000, 30000)])
        npg = max(1, min(npg, 4_000_000 // (g * qpg)))
        # below 5000 codes per group: the test function's workspace claim holds for the fused route only
        if npg >= 5000:
            npg = 4999
        return T.test_topk_inside_the_scoring_kernel, (rnd.choice([128, 128, 96, 256, 384, 512]), rnd.randint(0 if prod else 1, 4),
                                                       prod, g, qpg, npg, rnd.choice([1, 3, 10, 16, 17, 40, 64]))
    if kind == "split_q":
        return TS.test_quantize_split, (rnd.choice([32, 64, 96]), rnd.randint(0, 3), rnd.random() < 0.5, _n_at_128(rnd), rnd.random() < 0.5)
    if kind == "split_d":
        return TS.test_dequantize_split, (rnd.choice([32, 64, 96]), rnd.randint(0, 3), rnd.random() < 0.5, _n_at_128(rnd))
    d = rnd.choice([768, 1024, 1536, 3072])
    n = rnd.randint(1, 300 if d <= 1536 else 150)
    which = rnd.choice(["mse", "prod", "deq"])
    if which == "mse":
        return T.test_quantize_mse, (d, rnd.randint(1, 4), n, rnd.choice(["unit", "f32", "bf16"]))
    if which == "prod":
        return T.test_quantize_prod, (d, rnd.randint(0, 4), n, rnd.choice(["unit", "f32", "bf16"]))
    prod = rnd.random() < 0.5
    return T.test_dequantize, (d, rnd.randint(0 if prod else 1, 4), n, prod, rnd.random() < 0.5)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_valid_shapes_against_the_oracle(seed):
    rnd = random.Random(seed)
    for _ in range(60):
        fn, args = _draw(rnd)
        print(fn.__name__, args, flush=True)
        fn(*args)


# ------------------------------------------------------------------ padded rows, offset pointers, guard values


def _guarded(n_elems, dtype, off, tail=64):
    base = torch.full((off + n_elems + tail,), GUARD_I if dtype == torch.int32 else GUARD_F, dtype=dtype, device=DEV)
    return base, base[off: off + n_elems]


def _intact(base, off, n_elems, what):
    fill = GUARD_I if base.dtype == torch.int32 else GUARD_F
    assert bool((base[:off] == fill).all()) and bool((base[off + n_elems:] == fill).all()), f"{what}: written outside its rows"


def _shifted(t, off):
    """The same values at an address that is `off` elements past a fresh allocation (so less aligned)."""
    if t is None:
        return None
    base = torch.zeros(off + t.numel() + 8, dtype=t.dtype, device=DEV)
    v = base[off: off + t.numel()].view(t.shape)
    v.copy_(t)
    return v


def _quantize_padded(rnd):
    d = rnd.choice([128, 128, 128, 64, 96, 256, 512])
    prod = rnd.random() < 0.6
    bits = rnd.randint(0 if prod else 1, 4)
    n = _n_at_128(rnd) if d == 128 else rnd.randint(1, 600)
    bf16, normalise = rnd.random() < 0.5, rnd.random() < 0.7
    pad, xoff, woff = rnd.choice([0, 4, 8, 16, 40]), rnd.choice([0, 4, 8, 12]), rnd.choice([0, 0, 1, 2, 3, 4])
    mode = rnd.choice(["default", "default", "no images", "fp32 mfma"])
    print("quantize", d, bits, prod, n, bf16, normalise, pad, xoff, woff, mode, flush=True)
    p, Pi, S, c32, t32 = T.setup(d, bits, prod)
    x = W.unit_gaussian_rows(n, d, 1000 + n)
    if normalise:
        x = (x * np.exp(np.random.default_rng(n).normal(0, 1, (n, 1)))).astype(np.float32)
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    if bf16:
        xt = xt.to(torch.bfloat16)
    ld = d + pad
    xb = torch.zeros(xoff + n * ld + 64, dtype=xt.dtype, device=DEV)
    xv = xb[xoff: xoff + n * ld].view(n, ld)[:, :d]
    xv.copy_(xt)
    iw, qw = max(1, p.idx_words), p.qjl_words

    def run(xin, off):
        bi, idx = _guarded(n * iw, torch.int32, off)
        bq, qjl = _guarded(n * qw, torch.int32, off)
        bg, gamma = _guarded(n, torch.float32, off)
        bn, norm = _guarded(n, torch.float32, off)
        idx, qjl = idx.view(n, iw), qjl.view(n, qw)
        p.reserve(n, 0, 0)
        if prod:
            tq.tq_quantize_prod(p, xin, idx, qjl, gamma, norm if normalise else None)
        else:
            tq.tq_quantize_mse(p, xin, idx, norm if normalise else None)
        torch.cuda.synchronize()
        _intact(bi, off, n * iw if bits else 0, "idx")
        _intact(bq, off, n * qw if prod else 0, "qjl")
        _intact(bg, off, n if prod else 0, "gamma")
        _intact(bn, off, n if normalise else 0, "norm")
        return T.words(idx), T.words(qjl), gamma.cpu().numpy(), norm.cpu().numpy()

    a = run(xt.contiguous(), 0)
    if mode == "no images":
        p.drop_images()
    p.fp32_mfma = mode == "fp32 mfma"
    try:
        b = run(xv, woff)
    finally:
        p.fp32_mfma = False
        if mode == "no images":
            p.build_images()
    # the two calls may take different kernels: indices may differ inside the tie band, and what follows an
    # index (the residual, its norm, the sketch) is compared only where the indices agree
    same = True
    if bits:
        ia, ib = o.unpack_planes(a[0][:, : p.idx_words], bits, d), o.unpack_planes(b[0][:, : p.idx_words], bits, d)
        bad = int((ia != ib).sum())
        assert bad <= max(1, int(1e-4 * ia.size)), f"indices differ in {bad} of {ia.size}"
        same = bad == 0
    if prod and same:
        assert np.allclose(a[2], b[2], rtol=2e-5, atol=0), "gamma"
        za, zb = o.unpack_signs(a[1], d), o.unpack_signs(b[1], d)
        assert int((za != zb).sum()) <= max(1, int(1e-4 * za.size)), "signs"
    if normalise:
        assert np.allclose(a[3], b[3], rtol=4e-6, atol=0), "norm"


def _dequantize_padded(rnd):
    d = rnd.choice([128, 128, 128, 64, 96, 256, 512])
    prod = rnd.random() < 0.5
    bits = rnd.randint(0 if prod else 1, 4)
    n = _n_at_128(rnd) if d == 128 else rnd.randint(1, 600)
    pad, ooff, woff, with_norm = rnd.choice([0, 4, 8, 36]), rnd.choice([0, 4, 8]), rnd.choice([0, 0, 1, 2, 3, 4]), rnd.random() < 0.5
    mode = rnd.choice(["default", "default", "no images", "fp32 mfma"])
    print("dequantize", d, bits, prod, n, pad, ooff, woff, with_norm, mode, flush=True)
    p, Pi, S, c32, t32 = T.setup(d, bits, prod)
    c = T._random_codes(p, d, bits, prod, n, n + d)
    nm = c["norm"] if with_norm else None
    ld = d + pad
    ob, ov = _guarded(n * ld, torch.float32, ooff)
    dense = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, c["idx"], c["qjl"], c["gamma"], nm, dense)
    if mode == "no images":
        p.drop_images()
    p.fp32_mfma = mode == "fp32 mfma"
    try:
        tq.tq_dequantize(p, _shifted(c["idx"], woff), _shifted(c["qjl"], woff), _shifted(c["gamma"], woff), _shifted(nm, woff),
                         ov.view(n, ld)[:, :d])
    finally:
        p.fp32_mfma = False
        if mode == "no images":
            p.build_images()
    torch.cuda.synchronize()
    _intact(ob, ooff, n * ld, "x_out")
    full = ov.view(n, ld).cpu().numpy()
    assert np.all(full[:, d:] == GUARD_F), "x_out: the padding of a row was written"
    scale = (np.ones(n) if nm is None else nm.cpu().numpy().astype(np.float64))[:, None] / math.sqrt(d)
    P.check_close(full[:, :d], dense.cpu().numpy(), scale, "padded against dense dequantize", rel=2e-4)


def _score_padded(rnd):
    d = rnd.choice([128, 128, 128, 64, 96, 256, 384, 512, 768, 1536])
    prod = rnd.random() < 0.5
    bits = rnd.randint(0 if prod else 1, 4)
    g, qpg = rnd.choice([1, 2, 3, 8]), rnd.choice([1, 3, 4, 5, 32, 33, 70, 130, 260])
    npg = rnd.choice([rnd.randint(1, 300), rnd.randint(2040, 2060), rnd.randint(300, 9000)])
    npg = max(1, min(npg, 4_000_000 // (g * qpg), 8_000_000 // (g * d)))
    padq, pads = rnd.choice([0, 4, 12]), rnd.choice([0, 1, 2, 3, 4, 7, 64])
    woff, soff = rnd.choice([0, 0, 1, 2, 3, 4]), rnd.choice([0, 0, 1, 2, 4])
    topk = rnd.choice([0, 0, 5, 10, 16, 33])
    topk = topk if topk <= npg else 0
    mode = rnd.choice(["default", "fp32 mfma", "static scratch"])
    print("score", d, bits, prod, g, qpg, npg, padq, pads, woff, soff, topk, mode, flush=True)
    p, Pi, S, c32, t32 = T.setup(d, bits, prod)
    n, nq = g * npg, g * qpg
    c = T._random_codes(p, d, bits, prod, n, n + d)
    q = torch.from_numpy(W.gaussian_queries(nq, d, 3, unit=False)).to(DEV)
    qv = torch.zeros(nq * (d + padq) + 8, dtype=torch.float32, device=DEV)[: nq * (d + padq)].view(nq, d + padq)[:, :d]
    qv.copy_(q)
    dense = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
    p.reserve(n, nq, max(topk, 1))
    tq.tq_score(p, q, g, qpg, c["idx"], c["qjl"], c["gamma"], c["norm"], npg, dense)
    lds = npg + pads
    sb, sv = _guarded(nq * lds, torch.float32, soff)
    tb, ti = _guarded(nq * max(1, topk), torch.int32, woff)
    vb, tv = _guarded(nq * max(1, topk), torch.float32, woff)
    ti, tv = ti.view(nq, max(1, topk)), tv.view(nq, max(1, topk))
    codes = [_shifted(c[k], woff) for k in ("idx", "qjl", "gamma", "norm")]
    call = tq.tq_score
    if mode == "static scratch":
        p_need = tq.api._lib.load().tq_score_workspace_bytes(tq.api.C.byref(p.c), g, qpg, npg, int(prod), 1, topk)
        if 0 < p_need <= tq.tq_score_static_scratch_bytes():
            call = tq.tq_score_static
    p.fp32_mfma = mode == "fp32 mfma"
    try:
        call(p, qv, g, qpg, *codes, npg, sv.view(nq, lds)[:, :npg], topk, ti if topk else None, tv if topk else None)
    finally:
        p.fp32_mfma = False
    torch.cuda.synchronize()
    _intact(sb, soff, nq * lds, "scores")
    full = sv.view(nq, lds).cpu().numpy()
    assert np.all(full[:, npg:] == GUARD_F), "scores: the padding of a row was written"
    qn, nm = np.linalg.norm(q.cpu().numpy().astype(np.float64), axis=1), c["norm"].cpu().numpy()
    scale = np.concatenate([qn[i * qpg:(i + 1) * qpg, None] * nm[None, i * npg:(i + 1) * npg] for i in range(g)])
    P.check_close(full[:, :npg], dense.cpu().numpy(), scale, "padded against dense score", rel=2e-4)
    if topk:
        _intact(tb, woff, nq * topk, "topk_idx")
        _intact(vb, woff, nq * topk, "topk_val")
        assert np.array_equal(ti.cpu().numpy(), o.topk(full[:, :npg], topk)), "top-k against the call's own scores"


def _append_strided(rnd):
    d = 128
    prod = rnd.random() < 0.6
    bits = rnd.randint(0 if prod else 1, 4)
    n = rnd.choice([1, 2, 8, rnd.randint(1, 300), rnd.randint(1000, 4000)])
    first, step, bf16 = rnd.randint(0, 50), rnd.choice([1, 1, 2, 7, 100]), rnd.random() < 0.5
    if n * step > 100_000:
        step = 1
    rows = first + (n - 1) * step + 1 + rnd.randint(0, 5)
    print("append", bits, prod, n, first, step, bf16, flush=True)
    p, Pi, S, c32, t32 = T.setup(d, bits, prod)
    x = (W.unit_gaussian_rows(n, d, 2000 + n) * np.exp(np.random.default_rng(n).normal(0, 1, (n, 1)))).astype(np.float32)
    xt = torch.from_numpy(x).to(DEV)
    if bf16:
        xt = xt.to(torch.bfloat16)
    iw, qw = max(1, p.idx_words), p.qjl_words
    idx = torch.full((rows, iw), GUARD_I, dtype=torch.int32, device=DEV)
    qjl = torch.full((rows, qw), GUARD_I, dtype=torch.int32, device=DEV)
    gamma = torch.full((rows,), GUARD_F, dtype=torch.float32, device=DEV)
    norm = torch.full((rows,), GUARD_F, dtype=torch.float32, device=DEV)
    tq.tq_append(p, xt, idx if bits else None, qjl if prod else None, gamma if prod else None, norm, first, step)
    di, dq = torch.zeros((n, iw), dtype=torch.int32, device=DEV), torch.zeros((n, qw), dtype=torch.int32, device=DEV)
    dg, dn = torch.zeros(n, dtype=torch.float32, device=DEV), torch.zeros(n, dtype=torch.float32, device=DEV)
    if prod:
        tq.tq_quantize_prod(p, xt, di, dq, dg, dn)
    else:
        tq.tq_quantize_mse(p, xt, di, dn)
    torch.cuda.synchronize()
    sel = torch.arange(n, device=DEV) * step + first
    other = torch.ones(rows, dtype=torch.bool, device=DEV)
    other[sel] = False
    assert bool((norm[other] == GUARD_F).all()) and bool((idx[other] == GUARD_I).all()), "rows outside the append were written"
    assert bool((qjl[other] == GUARD_I).all()) and bool((gamma[other] == GUARD_F).all()), "rows outside the append were written"
    assert np.allclose(norm[sel].cpu().numpy(), dn.cpu().numpy(), rtol=4e-6), "norm"
    same = True
    if bits:
        ia, ib = o.unpack_planes(T.words(idx[sel]), bits, d), o.unpack_planes(T.words(di), bits, d)
        bad = int((ia != ib).sum())
        assert bad <= max(1, int(1e-4 * ia.size)), f"appended indices differ in {bad} of {ia.size}"
        same = bad == 0
    if prod and same:
        assert np.allclose(gamma[sel].cpu().numpy(), dg.cpu().numpy(), rtol=2e-5), "gamma"
        za, zb = o.unpack_signs(T.words(qjl[sel]), d), o.unpack_signs(T.words(dq), d)
        assert int((za != zb).sum()) <= max(1, int(1e-4 * za.size)), "signs"


@pytest.mark.parametrize("seed", [21, 22])
def test_padded_rows_offset_pointers_and_guard_values(seed):
    rnd = random.Random(seed)
    for _ in range(80):
        rnd.choice([_quantize_padded, _dequantize_padded, _score_padded, _append_strided])(rnd)
