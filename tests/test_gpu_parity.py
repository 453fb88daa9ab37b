"""GPU parity tests: every C-ABI entry point against the CPU oracle on the same
seeded inputs.  Sizes here are small enough for the oracle to finish in
seconds yet span several 128-row tiles and ragged tails."""
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


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def bf16_tensor(bits_u16):
    return torch.as_tensor(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16).to(DEV)


_cache = {}


def setup(d, bits_mse, prod, seed_pi=100, seed_s=200):
    key = (d, bits_mse, prod, seed_pi, seed_s)
    if key not in _cache:
        Pi = o.rotation_from_gaussian(W.gaussian_matrix(d, seed_pi))
        S = W.sketch_matrix(d, seed_s) if prod else None
        c32, t32, _ = o.codebook_fp32(d, bits_mse)
        p = tq.Params(d, bits_mse, torch.from_numpy(Pi), None if S is None else torch.from_numpy(S), c32, t32)
        _cache[key] = (p, Pi, S, c32, t32)
    return _cache[key]


def words(t):
    return t.cpu().numpy().view(np.uint32)


# ------------------------------------------------------------------ setup


def test_library_codebook_equals_oracle_tables():
    for d, b in [(128, 2), (128, 3), (1536, 4), (3072, 1)]:
        c, t, cost = tq.tq_build_codebook(d, b)
        c32, t32, cost_o = o.codebook_fp32(d, b)
        assert np.array_equal(c, c32) and np.array_equal(t, t32) and abs(cost / cost_o - 1) < 1e-8


@pytest.mark.parametrize("d", [64, 128, 352])
def test_derived_parameters(d):
    p, Pi, S, _, _ = setup(d, 2, True)
    torch.cuda.synchronize()
    assert np.array_equal(p.PiT.cpu().numpy(), Pi.T)
    assert np.array_equal(p.ST.cpu().numpy(), S.T)
    want = S.astype(np.float64) @ Pi.astype(np.float64).T
    P.check_close(p.SPiT.cpu().numpy(), want, np.linalg.norm(S, axis=1)[:, None] / math.sqrt(d), "S Pi^T", rel=2e-6)


# ------------------------------------------------------------------ codec stages (bit exact)


@pytest.mark.parametrize("d,bits,n", [(128, 2, 4096), (128, 1, 7), (96, 3, 129), (1536, 4, 513), (32, 4, 1),
                                      (3072, 1, 70), (160, 3, 1000)])
def test_stage_pack_bit_exact(d, bits, n):
    p, Pi, _, c32, t32 = setup(d, bits, False)
    x = W.unit_gaussian_rows(n, d, 40 + bits)
    y = o.rotate(x, Pi)
    # plant coordinates exactly on, just below and just above every boundary
    flat = y.reshape(-1)
    k = 0
    for t in t32:
        for v in (t, np.nextafter(t, np.float32(-1)), np.nextafter(t, np.float32(1))):
            flat[(k * 37) % flat.size] = v
            k += 1
    want = o.pack_planes(o.nearest_centroid(y, t32), bits)
    out = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
    tq.tq_stage_pack(p, dev(y), out)
    assert np.array_equal(words(out), want)


@pytest.mark.parametrize("d,n", [(128, 1000), (96, 3), (3072, 65)])
def test_stage_sign_pack_bit_exact(d, n):
    rng = np.random.default_rng(d + n)
    u = rng.standard_normal((n, d)).astype(np.float32)
    u.reshape(-1)[::17] = 0.0
    u.reshape(-1)[5::19] = -0.0
    out = torch.zeros((n, d // 32), dtype=torch.int32, device=DEV)
    tq.tq_stage_sign_pack(d, dev(u), out)
    assert np.array_equal(words(out), o.pack_signs(u >= 0))


@pytest.mark.parametrize("d,bits,n", [(128, 2, 777), (1536, 4, 130), (64, 3, 5), (128, 0, 9)])
def test_stage_unpack_exact(d, bits, n):
    p, _, _, c32, _ = setup(d, bits, False)
    rng = np.random.default_rng(bits)
    idx = rng.integers(0, 1 << bits, size=(n, d)).astype(np.int32)
    w = o.pack_planes(idx, bits)
    out = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    tq.tq_stage_unpack(p, dev(w.view(np.int32)) if bits else None, out)
    assert np.array_equal(out.cpu().numpy(), c32[idx])


# ------------------------------------------------------------------ quantize


def _quant_inputs(n, d, kind, seed):
    x = W.unit_gaussian_rows(n, d, seed)
    if kind == "unit":
        return x, dev(x), False
    if kind == "bf16unit":  # bf16 rows taken as they are (no normalisation, no norm stored)
        bits16 = W.f32_to_bf16_bits(x)
        return o.bf16_bits_to_f64(bits16), bf16_tensor(bits16), False
    x = (x.astype(np.float64) * np.exp(np.random.default_rng(seed).normal(0, 1.5, size=(n, 1)))).astype(np.float32)
    if n > 3:
        x[3] = 0.0  # a zero vector
    if kind == "f32":
        return x, dev(x), True
    bits16 = W.f32_to_bf16_bits(x)
    return o.bf16_bits_to_f64(bits16), bf16_tensor(bits16), True


@pytest.mark.parametrize("d,bits,n,kind", [
    (128, 2, 4096, "unit"), (128, 1, 300, "f32"), (128, 3, 129, "bf16"), (128, 4, 1, "f32"),
    (256, 4, 515, "unit"), (96, 2, 257, "f32"), (1536, 4, 300, "unit"), (3072, 1, 140, "bf16"),
    (64, 0, 40, "f32"),
    # d = 128 above the small-batch threshold: the bf16-piece contraction (rows of Pi^T as queries)
    (128, 1, 30000, "f32"), (128, 4, 25000, "unit"), (128, 3, 40000, "bf16"),
    # large batches of bf16 vectors: the kernel on the bf16 matrix cores (blocks of 256 vectors, ragged tails)
    (128, 1, 33000, "bf16"), (128, 2, 32845, "bf16unit"), (128, 4, 70001, "bf16"),
    # large batches of fp32 vectors: the same kernel on two pieces of x (five piece products)
    (128, 2, 33001, "f32"), (128, 3, 40000, "unit"), (128, 4, 8193, "f32"),
    # just above the threshold of that kernel: one vector, and one wavefront's worth, in the last block
    (128, 2, 8193, "bf16"), (128, 3, 8225, "bf16"),
])
def test_quantize_mse(d, bits, n, kind):
    p, Pi, _, c32, t32 = setup(d, bits, False)
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 7 * d + bits)
    idx_or, nu_or, y_or = o.quant_mse(x_or, Pi, t32, normalise)
    idx = torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device=DEV)
    norm = torch.zeros(n, dtype=torch.float32, device=DEV) if normalise else None
    tq.tq_quantize_mse(p, x_dev, idx, norm)
    if bits:
        got = o.unpack_planes(words(idx)[:, : p.idx_words], bits, d)
        P.check_indices(got, idx_or, y_or, t32)
    if normalise:
        P.check_close(norm.cpu().numpy(), nu_or, 0.0, "norm", rel=2e-6)


@pytest.mark.parametrize("d,bits,n,kind", [(1536, 4, 1, "unit"), (1536, 4, 8, "f32"), (3072, 2, 64, "bf16"), (512, 3, 5, "f32"),
                                          (1024, 1, 33, "bf16unit"), (768, 4, 64, "unit"), (4096, 2, 3, "f32"), (544, 0, 7, "f32")])
def test_quantize_a_handful_of_long_vectors(d, bits, n, kind):
    """Up to 64 vectors at d >= 512 with a workspace at hand: y = Pi x by the matrix-vector kernel, then norm, decision
    and packing per vector; without a workspace the tiled contraction.  Both against the oracle."""
    p, Pi, _, c32, t32 = setup(d, bits, False)
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 13 * d + bits)
    idx_or, nu_or, y_or = o.quant_mse(x_or, Pi, t32, normalise)
    keep = (p.workspace, p.c.workspace, p.c.workspace_bytes)
    try:
        for with_workspace in (True, False):
            if with_workspace:
                p.reserve(n, 0, 0)
                assert p.c.workspace_bytes >= n * d * 4
            else:
                p.workspace, p.c.workspace, p.c.workspace_bytes = None, 0, 0
            idx = torch.full((n + 1, max(1, p.idx_words)), -5, dtype=torch.int32, device=DEV)
            norm = torch.full((n + 1,), -5.0, dtype=torch.float32, device=DEV) if normalise else None
            tq.tq_quantize_mse(p, x_dev, idx[:n], None if norm is None else norm[:n])
            assert bool((idx[n] == -5).all()) and (norm is None or float(norm[n]) == -5.0)
            if bits:
                P.check_indices(o.unpack_planes(words(idx[:n])[:, : p.idx_words], bits, d), idx_or, y_or, t32)
            if normalise:
                P.check_close(norm[:n].cpu().numpy(), nu_or, 0.0, "norm", rel=2e-6)
    finally:
        p.workspace, p.c.workspace, p.c.workspace_bytes = keep


@pytest.mark.parametrize("d,bits_mse,n,kind", [(1536, 1, 1, "unit"), (3072, 1, 8, "f32"), (512, 3, 64, "bf16"), (1024, 0, 5, "f32"),
                                              (768, 4, 33, "unit"), (2048, 2, 2, "bf16unit"), (544, 2, 9, "f32")])
def test_quantize_prod_of_a_handful_of_long_vectors(d, bits_mse, n, kind):
    """Alg. 2 on the matrix-vector route (up to 64 vectors, d >= 512, workspace sized by tq_workspace_bytes)."""
    p, Pi, S, c32, t32 = setup(d, bits_mse, True)
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 17 * d + bits_mse)
    assert tq.tq_workspace_bytes(p, n, 0, 0) >= 2 * n * d * 4
    out = _run_prod(p, x_dev, n, normalise)
    _check_prod(p, Pi, S, c32, t32, x_or, normalise, *out)


def _run_prod(p, x_dev, n, normalise):
    idx = torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV)
    gamma = torch.zeros(n, dtype=torch.float32, device=DEV)
    norm = torch.zeros(n, dtype=torch.float32, device=DEV) if normalise else None
    p.reserve(n, 0, 0)
    tq.tq_quantize_prod(p, x_dev, idx, qjl, gamma, norm)
    return idx, qjl, gamma, norm


def _check_prod(p, Pi, S, c32, t32, x_or, normalise, idx, qjl, gamma, norm):
    d, bits = p.d, p.bits_mse
    xh, nu_or = o.unit_normalise(x_or, normalise)
    y_or = o.rotate(xh, Pi)
    idx_or = o.nearest_centroid(y_or, t32)
    got = o.unpack_planes(words(idx)[:, : p.idx_words], bits, d) if bits else np.zeros_like(idx_or)
    if bits:
        P.check_indices(got, idx_or, y_or, t32)
    # downstream of the GPU's own indices (teacher forcing)
    r, gamma_or, u_or = o.residual_and_sketch(xh, got, Pi, S, c32)
    P.check_close(gamma.cpu().numpy(), gamma_or, 0.0, "gamma", rel=1e-5)
    s_norm = np.linalg.norm(S.astype(np.float64), axis=1)
    P.check_signs(o.unpack_signs(words(qjl), d), u_or, s_norm[None, :] * gamma_or[:, None])
    if normalise:
        P.check_close(norm.cpu().numpy(), nu_or, 0.0, "norm", rel=2e-6)
    return got, gamma_or


@pytest.mark.parametrize("d,bits_mse,n,kind", [
    (128, 2, 2000, "bf16"), (128, 3, 129, "f32"), (128, 1, 4096, "unit"), (128, 0, 100, "f32"),
    (256, 2, 300, "unit"), (1536, 1, 200, "unit"), (96, 4, 130, "f32"),
    # d = 128 above the small-batch threshold: the bf16-piece contraction (rows of Pi^T as queries)
    (128, 0, 26000, "f32"), (128, 1, 33000, "unit"), (128, 4, 25001, "bf16"),
    # large batches of bf16 vectors: the kernel on the bf16 matrix cores (blocks of 256 vectors, ragged tails)
    (128, 0, 33000, "bf16"), (128, 1, 40001, "bf16"), (128, 2, 66000, "bf16"), (128, 3, 32768, "bf16unit"),
    (128, 4, 33333, "bf16"), (128, 2, 8193, "bf16"), (128, 1, 8449, "bf16"),
    # large batches of fp32 vectors: the same kernel on two pieces of x (five piece products)
    (128, 2, 33001, "f32"), (128, 3, 66000, "f32"), (128, 4, 9000, "unit"),
    # fp32 vectors and a small residual (gamma ~ 0.1 at 4 bits): two pieces of x would move gamma by more than
    # 1e-5 of itself, so these stay on the fp32 instructions
    (128, 4, 37512, "unit"), (128, 4, 25848, "f32"), (96, 4, 573, "unit"), (64, 4, 471, "f32"), (32, 4, 444, "f32"),
    (32, 3, 500, "f32"), (64, 3, 700, "unit"),
])
def test_quantize_prod(d, bits_mse, n, kind):
    p, Pi, S, c32, t32 = setup(d, bits_mse, True)
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 11 * d + bits_mse)
    out = _run_prod(p, x_dev, n, normalise)
    _check_prod(p, Pi, S, c32, t32, x_or, normalise, *out)


def test_both_arithmetic_paths_of_large_bf16_batches():
    """Large bf16 batches at d = 128 run on the bf16 matrix cores (exact pieces); TQ_FLAG_FP32_MFMA in the parameters keeps them on the
    fp32 matrix instructions.  Both must meet the oracle, and they must agree with each other on nearly every
    index and sign."""
    d, bits_mse, n = 128, 2, 34000
    p, Pi, S, c32, t32 = setup(d, bits_mse, True)
    x_or, x_dev, normalise = _quant_inputs(n, d, "bf16", 77)
    pieces = _run_prod(p, x_dev, n, normalise)
    _check_prod(p, Pi, S, c32, t32, x_or, normalise, *pieces)
    xt = [torch.zeros((n, d), dtype=torch.float32, device=DEV) for _ in range(2)]
    p.fp32_mfma = True
    try:
        plain = _run_prod(p, x_dev, n, normalise)
        tq.tq_dequantize(p, *plain, xt[0])
    finally:
        p.fp32_mfma = False  # the parameter object is shared with other tests
    _check_prod(p, Pi, S, c32, t32, x_or, normalise, *plain)
    same_idx = (words(pieces[0]) == words(plain[0])).mean()
    same_qjl = (words(pieces[1]) == words(plain[1])).mean()
    assert same_idx >= 0.9999 and same_qjl >= 0.999, (same_idx, same_qjl)
    tq.tq_dequantize(p, *plain, xt[1])
    nu = plain[3].cpu().numpy().astype(np.float64)
    P.check_close(xt[1].cpu().numpy(), xt[0].cpu().numpy().astype(np.float64), nu[:, None] / np.sqrt(d), "dequantize, pieces vs fp32")


@pytest.mark.parametrize("d,bits_mse,prod,kind,n", [(128, 2, True, "bf16", 20077), (128, 3, False, "bf16", 20077),
                                                    (128, 1, True, "bf16", 20077), (128, 4, True, "bf16", 20077),
                                                    (256, 2, True, "f32", 3000), (1536, 4, False, "unit", 700),
                                                    (96, 1, True, "bf16", 2500), (512, 3, True, "bf16", 1111)])
def test_parameter_images_change_nothing(d, bits_mse, prod, kind, n):
    """tq_build_images only moves the splitting of the matrices out of the kernels: with and without params.images
    the large-batch d = 128 kernels and the generic quantiser must write the same bits."""
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    want = (5 + 4) * 128 * 128 * 2 if d == 128 else 10 * d * d
    assert p.c.images != 0 and tq.tq_images_bytes(d) == p.images.numel() == want
    assert tq.tq_images_bytes(100) == 0
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 5)
    out = []
    try:
        for with_images in (True, False):
            if not with_images:
                p.drop_images()
            if prod:
                codes = _run_prod(p, x_dev, n, normalise)
            else:
                idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
                norm = torch.zeros(n, dtype=torch.float32, device=DEV) if normalise else None
                p.reserve(n, 0, 0)
                tq.tq_quantize_mse(p, x_dev, idx, norm)
                codes = (idx, None, None, norm)
            xt = torch.zeros((n, d), dtype=torch.float32, device=DEV)
            tq.tq_dequantize(p, *codes, xt)
            out.append([t.cpu().numpy() for t in (*codes, xt) if t is not None])
    finally:
        p.build_images()  # the parameter object is shared with other tests
    for a, b in zip(*out):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("d,bits_mse,n,kind", [(256, 2, 3000, "f32"), (512, 4, 1500, "unit"), (96, 1, 2500, "bf16")])
def test_both_arithmetic_paths_at_other_dimensions(d, bits_mse, n, kind):
    """Every d other than 128 runs the quantiser's contractions, many-query scoring and dequantisation on the bf16
    matrix cores (pieces); TQ_FLAG_FP32_MFMA in the parameters keeps them on the fp32 matrix instructions.  Both must meet the oracle
    and agree with each other."""
    p, Pi, S, c32, t32 = setup(d, bits_mse, True)
    x_or, x_dev, normalise = _quant_inputs(n, d, kind, 91)
    nq = 40  # more than 32 queries per group: the many-query kernel
    q = W.gaussian_queries(nq, d, 5, unit=False)
    p.reserve(n, nq, 0)

    def run():
        codes = _run_prod(p, x_dev, n, normalise)
        _check_prod(p, Pi, S, c32, t32, x_or, normalise, *codes)
        xt = torch.zeros((n, d), dtype=torch.float32, device=DEV)
        tq.tq_dequantize(p, *codes, xt)
        sc = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
        tq.tq_score(p, dev(q), 1, nq, *codes, n, sc)
        return codes, xt, sc

    pieces = run()
    p.fp32_mfma = True
    try:
        plain = run()
    finally:
        p.fp32_mfma = False  # the parameter object is shared with other tests
    # coordinate by coordinate (a word holds 32 of them): the two paths round differently, so a coordinate within
    # rounding of a cell boundary, or a sketch entry within rounding of zero, may fall on either side
    same = o.unpack_planes(words(pieces[0][0]), bits_mse, d) == o.unpack_planes(words(plain[0][0]), bits_mse, d)
    assert same.mean() >= 0.99999, same.mean()
    # signs only where the whole index vector agrees: one differing index changes that vector's residual
    rows = same.all(axis=1)
    assert rows.mean() > 0.99
    assert (o.unpack_signs(words(pieces[0][1]), d) == o.unpack_signs(words(plain[0][1]), d))[rows].mean() >= 0.9999
    # the same codes through both arithmetic paths
    xt2 = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    sc2 = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, *plain[0], xt2)
    tq.tq_score(p, dev(q), 1, nq, *plain[0], n, sc2)
    nu = plain[0][3].cpu().numpy().astype(np.float64) if normalise else np.ones(n)
    P.check_close(xt2.cpu().numpy(), plain[1].cpu().numpy().astype(np.float64), nu[:, None] / np.sqrt(d), "dequantize, pieces vs fp32")
    qn = np.linalg.norm(q.astype(np.float64), axis=1)
    P.check_close(sc2.cpu().numpy(), plain[2].cpu().numpy().astype(np.float64), qn[:, None] * nu[None, :], "scores, pieces vs fp32")


def test_large_batches_respect_row_strides_and_leave_the_tail_alone():
    """The large-batch kernels at d = 128 with padded input and output rows, a batch that ends inside a block of
    256, and guard rows behind every output that must stay untouched."""
    d, bits_mse, n, pad = 128, 2, 32768 + 300, 5
    p, Pi, S, c32, t32 = setup(d, bits_mse, True)
    x_or, x_dev, normalise = _quant_inputs(n, d, "bf16", 78)
    dense = _run_prod(p, x_dev, n, normalise)
    wide = torch.full((n, d + 64), 7.0, dtype=torch.bfloat16, device=DEV)
    wide[:, :d] = x_dev
    idx = torch.full((n + pad, p.idx_words), -1, dtype=torch.int32, device=DEV)
    qjl = torch.full((n + pad, p.qjl_words), -1, dtype=torch.int32, device=DEV)
    gamma = torch.full((n + pad,), -2.0, dtype=torch.float32, device=DEV)
    norm = torch.full((n + pad,), -2.0, dtype=torch.float32, device=DEV)
    tq.tq_quantize_prod(p, wide[:, :d], idx[:n], qjl[:n], gamma[:n], norm[:n])
    for got, want, fill in ((idx, dense[0], -1), (qjl, dense[1], -1), (gamma, dense[2], -2.0), (norm, dense[3], -2.0)):
        assert torch.equal(got[:n], want), "padded input rows change the codes"
        assert bool((got[n:] == fill).all()), "rows past the batch were written"
    out = torch.full((n + pad, d + 32), -3.0, dtype=torch.float32, device=DEV)
    ref = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, *dense, ref)
    tq.tq_dequantize(p, *dense, out[:n, :d])
    assert torch.equal(out[:n, :d], ref), "padded output rows change the values"
    assert bool((out[:n, d:] == -3.0).all()) and bool((out[n:] == -3.0).all()), "bytes outside the rows were written"


@pytest.mark.parametrize("bits_mse,prod,n,offset,pad", [(2, True, 300, 4, 0), (3, False, 9000, 0, 4), (1, True, 8300, 12, 4),
                                                        (4, False, 40, 4, 8)])
def test_bf16_rows_that_are_only_8_byte_aligned(bits_mse, prod, n, offset, pad):
    """bf16 rows need 8-byte alignment only; at d = 128 such rows take the kernel written for every dimension,
    which must not be handed the parameter images of the d = 128 kernels (they are built by default)."""
    d = 128
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    assert p.images is not None
    x_or, x_dev, normalise = _quant_inputs(n, d, "bf16", 3 * n + bits_mse)
    ld = d + pad
    buf = torch.zeros(offset + n * ld + 8, dtype=torch.bfloat16, device=DEV)
    xv = buf[offset: offset + n * ld].view(n, ld)[:, :d]
    xv.copy_(x_dev)
    assert xv.data_ptr() % 16 != 0 or (ld * 2) % 16 != 0
    if prod:
        out = _run_prod(p, xv, n, normalise)
        _check_prod(p, Pi, S, c32, t32, x_or, normalise, *out)
    else:
        idx_or, nu_or, y_or = o.quant_mse(x_or, Pi, t32, normalise)
        idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
        norm = torch.zeros(n, dtype=torch.float32, device=DEV)
        tq.tq_quantize_mse(p, xv, idx, norm)
        P.check_indices(o.unpack_planes(words(idx), bits_mse, d), idx_or, y_or, t32)
        P.check_close(norm.cpu().numpy(), nu_or, 0.0, "norm", rel=2e-6)


def test_quantize_is_deterministic_and_respects_row_stride():
    d, n = 128, 1000
    p, Pi, S, c32, t32 = setup(d, 2, True)
    x = W.unit_gaussian_rows(n, d, 5)
    xd = dev(x)
    a = _run_prod(p, xd, n, True)
    b = _run_prod(p, xd, n, True)
    for u, v in zip(a, b):
        assert torch.equal(u, v)
    wide = torch.zeros((n, d + 64), dtype=torch.float32, device=DEV)
    wide[:, :d] = xd
    idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV)
    gamma = torch.zeros(n, dtype=torch.float32, device=DEV)
    norm = torch.zeros(n, dtype=torch.float32, device=DEV)
    import ctypes as C
    from paper_2504_19874_amd import _lib
    st = _lib.load().tq_quantize_prod(C.byref(p.c), wide.data_ptr(), 0, n, d + 64, idx.data_ptr(), qjl.data_ptr(),
                                      gamma.data_ptr(), norm.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == 0
    assert torch.equal(idx, a[0]) and torch.equal(qjl, a[1]) and torch.equal(gamma, a[2])


def test_empty_and_error_paths():
    d = 128
    p, *_ = setup(d, 2, True)
    e = torch.zeros((0, d), dtype=torch.float32, device=DEV)
    tq.tq_quantize_mse(p, e, torch.zeros((0, p.idx_words), dtype=torch.int32, device=DEV), None)
    tq.tq_dequantize(p, torch.zeros((0, p.idx_words), dtype=torch.int32, device=DEV), None, None, None, e)
    # the two-pass path (any d other than 128) needs a residual workspace
    d2 = 256
    q, *_ = setup(d2, 2, True)
    with pytest.raises(tq.TurboQuantError, match="WORKSPACE"):
        p2 = tq.Params(d2, 2, q.Pi, q.S, q.centroids, q.bounds)
        x = dev(W.unit_gaussian_rows(8, d2, 1))
        tq.tq_quantize_prod(p2, x, torch.zeros((8, 16), dtype=torch.int32, device=DEV),
                            torch.zeros((8, 8), dtype=torch.int32, device=DEV),
                            torch.zeros(8, dtype=torch.float32, device=DEV), None)


# ------------------------------------------------------------------ dequantize / score / top-k


@pytest.mark.parametrize("d,bits_mse,n,prod,with_norm", [
    (128, 2, 1000, True, True), (128, 4, 129, False, False), (256, 3, 260, True, False),
    (1536, 4, 150, False, True), (128, 0, 64, True, True), (96, 1, 131, True, True),
    # d = 128 above the small-batch threshold: the bf16-piece contraction (rows of Pi^T as queries)
    (128, 2, 30000, True, True), (128, 3, 25000, False, False), (128, 0, 26001, True, True), (128, 4, 24600, False, True),
    (128, 1, 8200, True, True), (128, 1, 9000, False, False), (128, 2, 8193, True, False),
    # a handful of long vectors: matrix-vector products
    (1536, 4, 1, False, True), (3072, 1, 8, True, True), (512, 3, 31, True, False), (1024, 0, 5, True, True),
    (768, 2, 64, False, False), (544, 1, 3, True, True), (3584, 2, 2, True, True), (2048, 3, 13, False, True),
])
def test_dequantize(d, bits_mse, n, prod, with_norm):
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    rng = np.random.default_rng(d + n)
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool)
    gamma = rng.uniform(0.05, 0.6, size=n).astype(np.float32)
    norm = np.exp(rng.normal(0, 1, size=n)).astype(np.float32) if with_norm else None
    idx_w = dev(o.pack_planes(idx, bits_mse).view(np.int32)) if bits_mse else None
    out = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    if prod:
        want = o.dequant_prod(idx, z, gamma, Pi, S, c32, norm)
        tq.tq_dequantize(p, idx_w, dev(o.pack_signs(z).view(np.int32)), dev(gamma), None if norm is None else dev(norm), out)
    else:
        want = o.dequant_mse(idx, Pi, c32, norm)
        tq.tq_dequantize(p, idx_w, None, None, None if norm is None else dev(norm), out)
    scale = (np.ones(n) if norm is None else norm.astype(np.float64))[:, None] / math.sqrt(d)
    P.check_close(out.cpu().numpy(), want, scale, "dequantized coordinate")


@pytest.mark.parametrize("d,bits_mse,prod,n_groups,qpg,npg,topk", [
    (128, 2, True, 8, 4, 1000, 0), (128, 2, False, 1, 64, 4096, 10), (128, 3, True, 2, 4, 129, 5),
    (256, 4, False, 1, 130, 300, 10), (1536, 4, False, 1, 33, 257, 10), (128, 0, True, 1, 7, 100, 3),
    # few queries per code: int8 path (bits <= 3, d <= 512) and the fp32 lane-per-key path (the rest)
    (384, 1, False, 2, 5, 130, 4), (512, 3, True, 1, 4, 2100, 0), (64, 2, True, 3, 2, 77, 0),
    (128, 4, True, 2, 4, 300, 0), (640, 2, True, 1, 3, 200, 0), (128, 2, True, 1, 32, 1100, 0),
    # d = 128 single-kernel path: every bit width, one workgroup exactly (2048 keys), a ragged tail, several
    # workgroups, query blocks that are not multiples of 4, a handful of keys
    (128, 1, False, 3, 5, 2048, 0), (128, 3, False, 1, 4, 4100, 0), (128, 4, False, 2, 2, 2049, 3),
    (128, 0, True, 2, 4, 2300, 0), (128, 1, True, 1, 1, 5, 0), (128, 3, True, 1, 9, 6000, 0),
    # many queries per code: the bf16-piece contraction (mse any width, prod up to one index bit); tiles of
    # 128 queries x 256 codes with ragged edges on both sides, several groups, d that is not a multiple of 128
    (3072, 1, True, 1, 100, 700, 10), (128, 0, True, 1, 70, 300, 0), (160, 3, False, 2, 129, 513, 4),
    (1536, 2, False, 1, 200, 300, 0), (96, 1, False, 1, 65, 1000, 0), (1536, 4, False, 1, 257, 1025, 10),
    (128, 1, True, 3, 33, 257, 0), (1536, 2, True, 1, 150, 700, 0), (128, 2, True, 1, 200, 3000, 6),
    (256, 4, True, 2, 70, 130, 0),
    # d = 256..512: preparation kernel + int8 scoring kernel
    (256, 2, True, 2, 4, 1500, 0), (256, 4, True, 1, 3, 600, 0), (512, 1, False, 1, 8, 700, 0),
    (384, 3, True, 1, 2, 300, 0), (512, 4, False, 1, 4, 1100, 5),
    # d = 128 single-kernel path with a grid that fills the chip: 2048 keys per workgroup (33 groups x 5
    # workgroups; codes requested rounds ahead) and 1024 (20 groups), every bit width, ragged last workgroup
    (128, 1, False, 33, 4, 8292, 0), (128, 0, True, 33, 3, 8292, 0), (128, 3, False, 33, 4, 8200, 5),
    (128, 4, True, 33, 2, 8292, 0), (128, 2, False, 33, 4, 8292, 0), (128, 1, True, 20, 4, 8292, 0),
    (128, 3, True, 20, 4, 8292, 0), (128, 4, False, 20, 4, 8292, 3),
    # few queries against long codes: the integer-matrix-core kernel, 512 coordinates per launch
    (1536, 4, False, 1, 4, 2100, 10), (3072, 1, True, 1, 1, 700, 0), (1024, 2, True, 2, 5, 1500, 0), (640, 3, True, 1, 16, 900, 5),
    (768, 0, True, 1, 3, 130, 0), (2048, 2, False, 3, 9, 257, 3), (1536, 3, True, 1, 13, 4100, 0),
])
def test_score_and_topk(d, bits_mse, prod, n_groups, qpg, npg, topk):
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    n, nq = n_groups * npg, n_groups * qpg
    rng = np.random.default_rng(d + npg)
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool)
    gamma = rng.uniform(0.05, 0.6, size=n).astype(np.float32)
    norm = np.exp(rng.normal(0, 1, size=n)).astype(np.float32)
    q = W.gaussian_queries(nq, d, 3, unit=False)
    xt = o.dequant_prod(idx, z, gamma, Pi, S, c32, norm) if prod else o.dequant_mse(idx, Pi, c32, norm)
    want = np.concatenate([o.score(q[g * qpg:(g + 1) * qpg], xt[g * npg:(g + 1) * npg]) for g in range(n_groups)])
    idx_w = dev(o.pack_planes(idx, bits_mse).view(np.int32)) if bits_mse else None
    qjl_w = dev(o.pack_signs(z).view(np.int32)) if prod else None
    scores = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
    ti = torch.zeros((nq, max(1, topk)), dtype=torch.int32, device=DEV)
    tv = torch.zeros((nq, max(1, topk)), dtype=torch.float32, device=DEV)
    p.reserve(n, nq, topk)
    tq.tq_score(p, dev(q), n_groups, qpg, idx_w, qjl_w, dev(gamma) if prod else None, dev(norm), npg, scores,
                topk, ti if topk else None, tv if topk else None)
    qn = np.linalg.norm(q.astype(np.float64), axis=1)
    scale = np.concatenate([qn[g * qpg:(g + 1) * qpg, None] * norm[None, g * npg:(g + 1) * npg] for g in range(n_groups)])
    got = scores.cpu().numpy()
    P.check_close(got, want, scale, "score")
    if topk:
        # exact against the GPU's own score matrix, tolerant against the oracle's
        ref = o.topk(got, topk)
        assert np.array_equal(ti.cpu().numpy(), ref)
        assert np.array_equal(tv.cpu().numpy(), np.take_along_axis(got, ref, axis=1))
        P.check_topk(ti.cpu().numpy(), want, topk, scale.max(axis=1))
        # top-k without a score buffer gives the same answer
        ti2 = torch.zeros_like(ti)
        tq.tq_score(p, dev(q), n_groups, qpg, idx_w, qjl_w, dev(gamma) if prod else None, dev(norm), npg, None,
                    topk, ti2, None)
        assert torch.equal(ti, ti2)


@pytest.mark.parametrize("d,bits_mse,prod", [(128, 2, True), (256, 3, False)])
def test_score_with_a_codebook_that_is_not_symmetric(d, bits_mse, prod):
    """The few-query int8 kernels assume c[K-1-v] = -c[v]; any other table must be routed to a
    kernel that does not, and still match the oracle."""
    _, Pi, S, c_sym, _ = setup(d, bits_mse, prod)
    c32 = (c_sym.astype(np.float64) + 0.003 * np.arange(c_sym.size) / math.sqrt(d)).astype(np.float32)
    t32 = ((c32[:-1].astype(np.float64) + c32[1:].astype(np.float64)) / 2).astype(np.float32)
    p = tq.Params(d, bits_mse, torch.from_numpy(Pi), None if S is None else torch.from_numpy(S), c32, t32)
    n, nq = 700, 4
    rng = np.random.default_rng(11)
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool)
    gamma = rng.uniform(0.05, 0.6, size=n).astype(np.float32)
    norm = np.exp(rng.normal(0, 1, size=n)).astype(np.float32)
    q = W.gaussian_queries(nq, d, 5, unit=False)
    xt = o.dequant_prod(idx, z, gamma, Pi, S, c32, norm) if prod else o.dequant_mse(idx, Pi, c32, norm)
    want = o.score(q, xt)
    scores = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
    p.reserve(n, nq, 0)
    tq.tq_score(p, dev(q), 1, nq, dev(o.pack_planes(idx, bits_mse).view(np.int32)),
                dev(o.pack_signs(z).view(np.int32)) if prod else None, dev(gamma) if prod else None, dev(norm), n, scores)
    scale = np.linalg.norm(q.astype(np.float64), axis=1)[:, None] * norm[None, :]
    P.check_close(scores.cpu().numpy(), want, scale, "score, asymmetric codebook")


def test_score_equals_inner_product_with_dequantized_vectors():
    d, n, nq = 128, 500, 9
    p, Pi, S, c32, t32 = setup(d, 2, True)
    x = W.kv_keys_chunk(0, 0, n, d, 2, W.kv_outlier_channels(8, d, 2))
    idx, qjl, gamma, norm = _run_prod(p, bf16_tensor(x), n, True)
    q = dev(W.gaussian_queries(nq, d, 3, unit=False))
    xt = torch.zeros((n, d), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, idx, qjl, gamma, norm, xt)
    s = torch.zeros((nq, n), dtype=torch.float32, device=DEV)
    p.reserve(n, nq, 0)
    tq.tq_score(p, q, 1, nq, idx, qjl, gamma, norm, n, s)
    want = q.double().cpu().numpy() @ xt.double().cpu().numpy().T
    scale = np.linalg.norm(q.cpu().numpy(), axis=1)[:, None] * norm.cpu().numpy()[None, :]
    P.check_close(s.cpu().numpy(), want, scale, "score vs <q, dequantized>")


def _random_codes(p, d, bits_mse, prod, n, seed):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool)
    return dict(idx=dev(o.pack_planes(idx, bits_mse).view(np.int32)) if bits_mse else None,
                qjl=dev(o.pack_signs(z).view(np.int32)) if prod else None,
                gamma=dev(rng.uniform(0.05, 0.6, size=n).astype(np.float32)) if prod else None,
                norm=dev(np.exp(rng.normal(0, 1, size=n)).astype(np.float32)))


def _topk_both_ways(p, q, n_groups, qpg, c, npg, topk):
    """tq_score with a score buffer and top-k, and top-k alone: the indices and values must be the stable
    descending sort of the score matrix the same call wrote (equal scores by lower index)."""
    nq = n_groups * qpg
    prod = c["qjl"] is not None
    scores = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
    ti = torch.full((nq, topk), -5, dtype=torch.int32, device=DEV)
    tv = torch.full((nq, topk), float("nan"), dtype=torch.float32, device=DEV)
    p.reserve_score(n_groups, qpg, npg, prod, True, topk)
    tq.tq_score(p, q, n_groups, qpg, c["idx"], c["qjl"], c["gamma"], c["norm"], npg, scores, topk, ti, tv)
    got = scores.cpu().numpy()
    k_real = min(topk, npg)
    ref = o.topk(got, k_real)
    assert np.array_equal(ti.cpu().numpy()[:, :k_real], ref)
    assert np.array_equal(tv.cpu().numpy()[:, :k_real], np.take_along_axis(got, ref, axis=1))
    if k_real < topk:  # more wanted than there are codes
        assert np.all(ti.cpu().numpy()[:, k_real:] == -1) and np.all(np.isneginf(tv.cpu().numpy()[:, k_real:]))
    # no score buffer: a workspace sized for exactly this call (no score matrix where the selection is fused)
    ti2 = torch.full_like(ti, -5)
    tv2 = torch.full_like(tv, float("nan"))
    p.workspace, p.c.workspace, p.c.workspace_bytes = None, 0, 0
    p.reserve_score(n_groups, qpg, npg, prod, False, topk)
    tq.tq_score(p, q, n_groups, qpg, c["idx"], c["qjl"], c["gamma"], c["norm"], npg, None, topk, ti2, tv2)
    assert torch.equal(ti, ti2) and torch.equal(tv, tv2)
    return got, p.workspace.numel()


@pytest.mark.parametrize("d,bits_mse,prod,n_groups,qpg,npg,topk", [
    (128, 2, False, 1, 300, 200000, 10),   # two query blocks x 128 ranges of several 256-code tiles
    (128, 1, True, 1, 130, 150001, 16),    # the list length limit; a ragged last tile
    (96, 3, True, 3, 70, 5000, 7),         # three groups (query blocks do not divide the XCD count), 128-code tiles
    (256, 4, False, 2, 257, 3000, 1),      # k = 1; query blocks with a ragged tail
    (128, 2, False, 1, 100, 5, 10),        # more wanted than there are codes
    (128, 3, False, 1, 90, 70000, 17),     # above the list length: the separate top-k kernel over a score matrix
    (128, 3, False, 1, 90, 8, 17),         # that kernel with more wanted than there are codes (a 16-byte aligned row)
    (128, 2, True, 2, 4, 6, 9),            # the same on the few-query route
])
def test_topk_inside_the_scoring_kernel(d, bits_mse, prod, n_groups, qpg, npg, topk):
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    n, nq = n_groups * npg, n_groups * qpg
    c = _random_codes(p, d, bits_mse, prod, n, d + npg)
    q = dev(W.gaussian_queries(nq, d, 3, unit=False))
    _, ws = _topk_both_ways(p, q, n_groups, qpg, c, npg, topk)
    if topk <= 16 and npg >= 5000:
        assert ws < nq * npg  # far below a score matrix (4 bytes per pair)


@pytest.mark.parametrize("d,bits_mse,prod,n_groups,qpg,npg,topk", [
    (128, 2, True, 2, 4, 70001, 10), (1536, 4, False, 1, 1, 66000, 64), (128, 1, False, 3, 33, 131072, 5),
    (256, 3, True, 1, 2, 65536, 1), (128, 4, False, 1, 128, 65537, 16),
])
def test_topk_over_a_few_long_rows(d, bits_mse, prod, n_groups, qpg, npg, topk):
    """Few queries against many codes: the rows of the score matrix are cut into chunks, one workgroup per (row,
    chunk), and the chunks' lists are joined; same answer as a stable sort of the scores the call wrote."""
    p, Pi, S, c32, t32 = setup(d, bits_mse, prod)
    c = _random_codes(p, d, bits_mse, prod, n_groups * npg, d + npg)
    q = dev(W.gaussian_queries(n_groups * qpg, d, 3, unit=False))
    _topk_both_ways(p, q, n_groups, qpg, c, npg, topk)
    # a workspace without room for the chunks' lists (sized as for a call without top-k): one workgroup per row
    # (few-query routes only: the many-query kernel's own selection cannot do without its lists)
    if qpg > 16:
        return
    nq = n_groups * qpg
    keep = (p.workspace, p.c.workspace, p.c.workspace_bytes)
    try:
        p.workspace, p.c.workspace, p.c.workspace_bytes = None, 0, 0
        p.reserve_score(n_groups, qpg, npg, prod, True, 0)
        scores = torch.zeros((nq, npg), dtype=torch.float32, device=DEV)
        ti = torch.full((nq, topk), -5, dtype=torch.int32, device=DEV)
        tq.tq_score(p, q, n_groups, qpg, c["idx"], c["qjl"], c["gamma"], c["norm"], npg, scores, topk, ti, None)
        assert np.array_equal(ti.cpu().numpy(), o.topk(scores.cpu().numpy(), topk))
    finally:
        p.workspace, p.c.workspace, p.c.workspace_bytes = keep


def test_topk_inside_the_scoring_kernel_on_adversarial_orders():
    """Every tile beats the previous one (scores grow with the code index), and every score equal (the k
    lowest indices win): the selection must not depend on the order in which tiles and ranges are met."""
    d, bits_mse, nq, n, topk = 128, 2, 140, 90000, 10
    p, Pi, S, c32, t32 = setup(d, bits_mse, False)
    one = np.random.default_rng(1).integers(0, 4, size=(1, d)).astype(np.int32)
    words1 = o.pack_planes(one, bits_mse).view(np.int32)
    idx = dev(np.repeat(words1, n, axis=0))
    q = dev(W.gaussian_queries(nq, d, 9, unit=False))
    grow = dict(idx=idx, qjl=None, gamma=None, norm=dev(np.linspace(1.0, 2.0, n).astype(np.float32)))
    got, _ = _topk_both_ways(p, q, 1, nq, grow, n, topk)
    assert (got[:, -1] > got[:, 0]).any() and (got[:, -1] < got[:, 0]).any()  # rising rows and falling rows
    flat = dict(idx=idx, qjl=None, gamma=None, norm=dev(np.ones(n, dtype=np.float32)))
    got, _ = _topk_both_ways(p, q, 1, nq, flat, n, topk)
    assert np.all(got == got[:, :1])
    # a block of exact ties that straddles tiles and ranges, in the middle of random codes
    c = _random_codes(p, d, bits_mse, False, n, 77)
    c["idx"][30000:52000] = idx[30000:52000]
    c["norm"][30000:52000] = 50.0
    _topk_both_ways(p, q, 1, nq, c, n, topk)
