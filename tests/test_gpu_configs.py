"""The five benchmark configurations at their full sizes, in the launch
configuration the benchmark uses.  Small ones are compared in full with the
oracle; the million-vector ones on their first 131072 rows in full (indices,
residual norms, signs, every score of every query, and the top-10 of every
query within that subset ranked on the oracle's scores), on sampled rows and
sampled (query, code) pairs from the whole set, plus properties that hold at
any size (top-k of the GPU's own score matrix)."""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import turboquant_oracle as o
from tests import parity as P
from tests.test_gpu_parity import DEV, bf16_tensor, dev, words

pytestmark = pytest.mark.gpu

tq = pytest.importorskip("paper_2504_19874_amd")


def params_for(cfg):
    Pi = o.rotation_from_gaussian(W.gaussian_matrix(cfg.d, cfg.seed_pi))
    S = W.sketch_matrix(cfg.d, cfg.seed_s) if cfg.kind == "prod" else None
    c32, t32, _ = o.codebook_fp32(cfg.d, cfg.bits_mse)
    p = tq.Params(cfg.d, cfg.bits_mse, torch.from_numpy(Pi), None if S is None else torch.from_numpy(S), c32, t32)
    return p, Pi, S, c32, t32


def alloc_codes(p, n, prod):
    idx = torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device=DEV)
    qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device=DEV) if prod else None
    gamma = torch.zeros(n, dtype=torch.float32, device=DEV) if prod else None
    return idx, qjl, gamma


def test_c1_mse_b2_d128_full():
    cfg = W.CONFIGS["C1"]
    p, Pi, _, c32, t32 = params_for(cfg)
    x = W.unit_gaussian_rows(cfg.n, cfg.d, cfg.seed_x)
    q = W.unit_gaussian_rows(cfg.nq, cfg.d, cfg.seed_q)
    idx, _, _ = alloc_codes(p, cfg.n, False)
    tq.tq_quantize_mse(p, dev(x), idx, None)
    idx_or, _, y_or = o.quant_mse(x, Pi, t32, normalise=False)
    got = o.unpack_planes(words(idx), cfg.bits, cfg.d)
    P.check_indices(got, idx_or, y_or, t32)
    xt = torch.zeros((cfg.n, cfg.d), dtype=torch.float32, device=DEV)
    tq.tq_dequantize(p, idx, None, None, None, xt)
    want = o.dequant_mse(got, Pi, c32)
    P.check_close(xt.cpu().numpy(), want, 1 / math.sqrt(cfg.d), "C1 dequantized")
    s = torch.zeros((cfg.nq, cfg.n), dtype=torch.float32, device=DEV)
    p.reserve(cfg.n, cfg.nq, 0)
    tq.tq_score(p, dev(q), 1, cfg.nq, idx, None, None, None, cfg.n, s)
    P.check_close(s.cpu().numpy(), o.score(q, want), 1.0, "C1 score")
    # the quantiser meets Theorem 1 on this data: D_mse ~ 0.116 at d = 128, b = 2
    D = np.mean(np.sum((x - xt.cpu().numpy()) ** 2, axis=1))
    assert abs(D - 0.116) < 0.003


def _kv_setup(cfg):
    keys = W.kv_keys(cfg.n_groups, cfg.n, cfg.d, cfg.seed_x).reshape(-1, cfg.d)
    q = W.gaussian_queries(cfg.nq, cfg.d, cfg.seed_q, unit=False)
    return keys, q


def _quantize_kv(p, keys_bits, n):
    idx, qjl, gamma = alloc_codes(p, n, True)
    norm = torch.zeros(n, dtype=torch.float32, device=DEV)
    p.reserve(n, 64, 0)
    tq.tq_quantize_prod(p, bf16_tensor(keys_bits), idx, qjl, gamma, norm)
    return idx, qjl, gamma, norm


def test_c2_kv_prod_b3_full():
    cfg = W.CONFIGS["C2"]
    p, Pi, S, c32, t32 = params_for(cfg)
    keys, _ = _kv_setup(cfg)
    n = keys.shape[0]
    idx, qjl, gamma, norm = _quantize_kv(p, keys, n)
    x_or = o.bf16_bits_to_f64(keys)
    xh, nu_or = o.unit_normalise(x_or)
    y_or = o.rotate(xh, Pi)
    idx_or = o.nearest_centroid(y_or, t32)
    got = o.unpack_planes(words(idx), cfg.bits_mse, cfg.d)
    frac = P.check_indices(got, idx_or, y_or, t32)
    _, gamma_or, u_or = o.residual_and_sketch(xh, got, Pi, S, c32)
    P.check_close(gamma.cpu().numpy(), gamma_or, 0.0, "C2 gamma", rel=1e-5)
    P.check_close(norm.cpu().numpy(), nu_or, 0.0, "C2 norm", rel=2e-6)
    s_norm = np.linalg.norm(S.astype(np.float64), axis=1)
    P.check_signs(o.unpack_signs(words(qjl), cfg.d), u_or, s_norm[None, :] * gamma_or[:, None])
    print(f"C2 index agreement {frac:.7f}")


@pytest.mark.parametrize("name", ["C3", "C3b4"])
def test_c3_decode_scoring_full(name):
    cfg = W.CONFIGS[name]
    p, Pi, S, c32, t32 = params_for(cfg)
    keys, q = _kv_setup(cfg)
    n = keys.shape[0]
    idx, qjl, gamma, norm = _quantize_kv(p, keys, n)
    scores = torch.zeros((cfg.nq, cfg.n), dtype=torch.float32, device=DEV)
    p.reserve(n, cfg.nq, 0)
    tq.tq_score(p, dev(q), cfg.n_groups, cfg.q_per_group, idx, qjl, gamma, norm, cfg.n, scores)
    got_idx = o.unpack_planes(words(idx), cfg.bits_mse, cfg.d)
    z = o.unpack_signs(words(qjl), cfg.d)
    g_np, nu_np = gamma.cpu().numpy(), norm.cpu().numpy()
    s_gpu = scores.cpu().numpy()
    qn = np.linalg.norm(q.astype(np.float64), axis=1)
    for g in range(cfg.n_groups):
        rows = slice(g * cfg.n, (g + 1) * cfg.n)
        xt = o.dequant_prod(got_idx[rows], z[rows], g_np[rows], Pi, S, c32, nu_np[rows])
        qs = slice(g * cfg.q_per_group, (g + 1) * cfg.q_per_group)
        P.check_close(s_gpu[qs], o.score(q[qs], xt), qn[qs, None] * nu_np[None, rows], f"{name} logits, head {g}")
    # the estimator is unbiased: over many keys the mean error is small against its spread
    xs = o.bf16_bits_to_f64(keys[: cfg.n])
    err = s_gpu[0] - q[0].astype(np.float64) @ xs.T
    assert abs(err.mean()) < 5 * err.std() / math.sqrt(cfg.n)


HEAD = 131072  # rows of the million-vector sets that the oracle takes in full


def _ann_database(cfg, p, prod):
    """Generate on the host in chunks, upload, quantise everything; keep the
    first HEAD rows and a sample of the others on the host for the oracle."""
    n, d = cfg.n, cfg.d
    x_head = np.empty((HEAD, d), dtype=np.float32)
    x_dev = torch.empty((n, d), dtype=torch.float32, device=DEV)
    rng = np.random.default_rng(99)
    sample = np.unique(np.concatenate([np.arange(0, 300), np.arange(n - 300, n),
                                       rng.integers(0, n, size=1500)]))
    kept = {}
    for start, blk in W.mixture_rows(n, d, cfg.seed_x, cfg.seed_x):
        x_dev[start:start + blk.shape[0]] = torch.from_numpy(blk).to(DEV)
        sel = sample[(sample >= start) & (sample < start + blk.shape[0])]
        for i in sel:
            kept[int(i)] = blk[i - start].copy()
        if start < HEAD:
            x_head[start:min(HEAD, start + blk.shape[0])] = blk[:HEAD - start]
    x_s = np.stack([kept[int(i)] for i in sample])
    idx, qjl, gamma = alloc_codes(p, n, prod)
    # quantisation scratch, and exactly what the top-k call takes (no score matrix: the selection is fused)
    p.reserve(n, cfg.nq, 0).reserve_score(1, cfg.nq, n, prod, False, cfg.topk)
    assert p.workspace.numel() < (1 << 30)
    if prod:
        tq.tq_quantize_prod(p, x_dev, idx, qjl, gamma, None)
    else:
        tq.tq_quantize_mse(p, x_dev, idx, None)
    torch.cuda.synchronize()
    del x_dev
    return sample, x_s, idx, qjl, gamma, x_head


def _ann_score_checks(cfg, p, Pi, S, c32, idx, qjl, gamma, prod):
    n, d = cfg.n, cfg.d
    centers = W.mixture_centers(d, cfg.seed_x)
    q = W.mixture_chunk(0, cfg.nq, d, cfg.seed_q, centers)
    qd = dev(q)
    ti = torch.zeros((cfg.nq, cfg.topk), dtype=torch.int32, device=DEV)
    tv = torch.zeros((cfg.nq, cfg.topk), dtype=torch.float32, device=DEV)
    tq.tq_score(p, qd, 1, cfg.nq, idx, qjl, gamma, None, n, None, cfg.topk, ti, tv)
    # a slice of queries with the score matrix materialised
    nqs = 48
    s = torch.zeros((nqs, n), dtype=torch.float32, device=DEV)
    p.reserve_score(1, nqs, n, prod, True, 0)
    tq.tq_score(p, qd[:nqs], 1, nqs, idx, qjl, gamma, None, n, s)
    # the two calls rotate the queries with different kernels (few vs many queries), so the
    # scores agree to rounding, not bit for bit: compare the top-k with the tolerance rule
    s_np = s.cpu().numpy()
    P.check_topk(ti[:nqs].cpu().numpy(), s_np, cfg.topk, np.ones(nqs))
    ref_v, _ = torch.topk(s, cfg.topk, dim=1)
    P.check_close(tv[:nqs].cpu().numpy(), ref_v.cpu().numpy(), 1.0, "top-k values", rel=2e-6)
    # sampled (query, code) pairs against the oracle, including each query's winners
    rng = np.random.default_rng(5)
    cols = np.unique(np.concatenate([rng.integers(0, n, size=3000), ti[:nqs].cpu().numpy().ravel()]))
    cd = torch.as_tensor(cols, device=DEV)
    got_idx = o.unpack_planes(words(idx[cd]), cfg.bits_mse, d)
    if prod:
        xt = o.dequant_prod(got_idx, o.unpack_signs(words(qjl[cd]), d), gamma[cd].cpu().numpy(), Pi, S, c32)
    else:
        xt = o.dequant_mse(got_idx, Pi, c32)
    want = o.score(q[:nqs], xt)
    P.check_close(s[:, cd].cpu().numpy(), want, 1.0, f"{cfg.name} sampled scores")
    del s
    return q, ti


def _ann_head_checks(cfg, p, Pi, S, c32, q, idx, qjl, gamma, got_head, z_head, prod):
    """Every query against the first HEAD codes: all HEAD x nq scores against the oracle (fed the GPU's own
    codes), and the top-10 within that subset, selected by the library without a score buffer, judged on
    the ORACLE's scores."""
    d = cfg.d
    g_head = gamma[:HEAD].cpu().numpy() if prod else None
    xt = o.dequant_prod(got_head, z_head, g_head, Pi, S, c32) if prod else o.dequant_mse(got_head, Pi, c32)
    want = o.score(q, xt)  # [nq, HEAD] fp64
    del xt
    qd = dev(q)
    sub = (idx[:HEAD], qjl[:HEAD] if prod else None, gamma[:HEAD] if prod else None)
    s = torch.zeros((cfg.nq, HEAD), dtype=torch.float32, device=DEV)
    p.reserve_score(1, cfg.nq, HEAD, prod, True, 0)
    tq.tq_score(p, qd, 1, cfg.nq, *sub, None, HEAD, s)
    worst = P.check_close(s.cpu().numpy(), want, 1.0, f"{cfg.name} scores of the first {HEAD} codes")
    del s
    ti = torch.zeros((cfg.nq, cfg.topk), dtype=torch.int32, device=DEV)
    tv = torch.zeros((cfg.nq, cfg.topk), dtype=torch.float32, device=DEV)
    p.reserve_score(1, cfg.nq, HEAD, prod, False, cfg.topk)
    tq.tq_score(p, qd, 1, cfg.nq, *sub, None, HEAD, None, cfg.topk, ti, tv)
    ti_np = ti.cpu().numpy()
    P.check_topk(ti_np, want, cfg.topk, np.ones(cfg.nq))
    P.check_close(tv.cpu().numpy(), np.take_along_axis(want, ti_np.astype(np.int64), axis=1), 1.0,
                  f"{cfg.name} top-{cfg.topk} values")
    print(f"{cfg.name}: {cfg.nq} x {HEAD} scores within {worst:.3f} of the tolerance; top-{cfg.topk} of every query "
          f"agrees with the oracle's ranking")


def test_c4_ann_mse_b4_d1536_full():
    cfg = W.CONFIGS["C4"]
    p, Pi, _, c32, t32 = params_for(cfg)
    sample, x_s, idx, _, _, x_head = _ann_database(cfg, p, False)
    idx_or, _, y_or = o.quant_mse(x_s, Pi, t32, normalise=False)
    got = o.unpack_planes(words(idx[torch.as_tensor(sample, device=DEV)]), cfg.bits_mse, cfg.d)
    frac = P.check_indices(got, idx_or, y_or, t32)
    print(f"C4 index agreement on {sample.size} sampled rows {frac:.7f}")
    # the first HEAD rows in full
    idx_or, _, y_or = o.quant_mse(x_head, Pi, t32, normalise=False)
    got_head = o.unpack_planes(words(idx[:HEAD]), cfg.bits_mse, cfg.d)
    frac = P.check_indices(got_head, idx_or, y_or, t32)
    print(f"C4 index agreement on the first {HEAD} rows {frac:.7f}")
    del idx_or, y_or, x_head
    q, _ = _ann_score_checks(cfg, p, Pi, None, c32, idx, None, None, False)
    _ann_head_checks(cfg, p, Pi, None, c32, q, idx, None, None, got_head, None, False)


def test_c5_ann_prod_b2_d3072_full():
    cfg = W.CONFIGS["C5"]
    p, Pi, S, c32, t32 = params_for(cfg)
    sample, x_s, idx, qjl, gamma, x_head = _ann_database(cfg, p, True)
    sd = torch.as_tensor(sample, device=DEV)
    xh, _ = o.unit_normalise(x_s, False)
    y_or = o.rotate(xh, Pi)
    idx_or = o.nearest_centroid(y_or, t32)
    got = o.unpack_planes(words(idx[sd]), cfg.bits_mse, cfg.d)
    frac = P.check_indices(got, idx_or, y_or, t32)
    _, gamma_or, u_or = o.residual_and_sketch(xh, got, Pi, S, c32)
    P.check_close(gamma[sd].cpu().numpy(), gamma_or, 0.0, "C5 gamma", rel=1e-5)
    s_norm = np.linalg.norm(S.astype(np.float64), axis=1)
    fs = P.check_signs(o.unpack_signs(words(qjl[sd]), cfg.d), u_or, s_norm[None, :] * gamma_or[:, None])
    print(f"C5 index agreement {frac:.7f}, sign agreement {fs:.7f} on {sample.size} sampled rows")
    # the first HEAD rows in full
    xh, _ = o.unit_normalise(x_head, False)
    del x_head
    y_or = o.rotate(xh, Pi)
    idx_or = o.nearest_centroid(y_or, t32)
    got_head = o.unpack_planes(words(idx[:HEAD]), cfg.bits_mse, cfg.d)
    frac = P.check_indices(got_head, idx_or, y_or, t32)
    del y_or, idx_or
    _, gamma_or, u_or = o.residual_and_sketch(xh, got_head, Pi, S, c32)
    del xh
    P.check_close(gamma[:HEAD].cpu().numpy(), gamma_or, 0.0, "C5 gamma", rel=1e-5)
    z_head = o.unpack_signs(words(qjl[:HEAD]), cfg.d)
    fs = P.check_signs(z_head, u_or, s_norm[None, :] * gamma_or[:, None])
    del u_or
    print(f"C5 index agreement {frac:.7f}, sign agreement {fs:.7f} on the first {HEAD} rows")
    q, _ = _ann_score_checks(cfg, p, Pi, S, c32, idx, qjl, gamma, True)
    _ann_head_checks(cfg, p, Pi, S, c32, q, idx, qjl, gamma, got_head, z_head, True)
