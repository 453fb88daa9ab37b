"""The GPU path against what the paper's theorems fix (no oracle involved), and the
recall harness against the oracle on a case small enough for it."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2504_19874_amd as tq
import workloads as W
from oracle import turboquant_oracle as o
from paper_2504_19874_amd import recall as R

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d", [128, 1536])
def test_distortions_match_theorems_1_and_2(d):
    """D_mse = d * C(f_X, b) (Theorem 1's proof: the per-coordinate Lloyd-Max cost, summed);
    D_prod of the two-stage quantiser = pi/(2d) * d * C(f_X, b-1) * ||y||^2 (Theorem 2's proof);
    the MSE quantiser's inner products shrink by 2/pi at b = 1 (Sec. 3.2) while the two-stage
    estimator is unbiased; everything lies between the bounds of Theorem 3 and Theorems 1/2."""
    n, nq = 20000, 200
    for bits in (1, 2, 3, 4):
        cost = tq.tq_build_codebook(d, bits)[2]
        m = R.distortion(tq, torch, W, d, n, nq, bits, "mse")
        assert abs(m["D_mse"] / (d * cost) - 1) < 0.02
        assert m["lower_mse"] < m["D_mse"] < m["upper_mse"]
        cost_prev = tq.tq_build_codebook(d, bits - 1)[2]
        p = R.distortion(tq, torch, W, d, n, nq, bits, "prod")
        assert abs(p["D_prod"] / (math.pi / (2 * d) * d * cost_prev) - 1) < 0.05
        assert p["lower_prod"] < p["D_prod"] < p["upper_prod"]
        assert abs(p["slope"] - 1) < 0.01 and abs(p["bias"]) < 0.005 * math.sqrt(p["D_prod"])
        if bits == 1:
            assert abs(m["slope"] - 2 / math.pi) < 0.01


def test_entropy_of_the_stored_indices():
    """Sec. 3.1: at b = 4 the indices carry about 3.8 bits each (a 5 % saving for an entropy coder);
    the histogram of what the library stores must be the codebook's bucket probabilities."""
    d, n, bits = 1536, 4000, 4
    got = R.index_entropy(tq, torch, W, d, n, bits)
    c, _, _ = o.lloyd_max_codebook(d, bits)
    p = o.bucket_masses(c, d)
    assert np.max(np.abs(np.array(got["freq"]) - p)) < 2e-3
    assert abs(got["entropy_bits"] - float(-np.sum(p * np.log2(p)))) < 0.01
    assert abs(got["entropy_bits"] - 3.8) < 0.05 and abs(got["saving"] - 0.05) < 0.01


@pytest.mark.parametrize("d,bits", [(1536, 4), (128, 3)])
def test_prefix_code_on_what_the_gpu_stores(d, bits):
    """Sec. 3.1, entropy-coding paragraph, end to end: indices quantised on the GPU, coded with the library's prefix
    code for the codebook's bucket probabilities, decode to the same words; the stream has the length the oracle's
    code lengths predict for these indices and, at b = 4, saves the 5 % the paper quotes."""
    from paper_2504_19874_amd import entropy as E
    n = 3000
    c, t, _ = tq.tq_build_codebook(d, bits)
    p = tq.make_params(d, bits, W.gaussian_matrix(d, 31))
    x = torch.from_numpy(W.unit_gaussian_rows(n, d, 32)).cuda()
    idx = torch.zeros((n, p.idx_words), dtype=torch.int32, device="cuda")
    p.reserve(n, 0, 0)
    tq.tq_quantize_mse(p, x, idx, None)
    words = idx.cpu().numpy().view(np.uint32)
    masses = E.bucket_masses(d, bits, c)
    code = E.PrefixCode(masses)
    stream, offs = code.encode(words, d)
    assert np.array_equal(code.decode(stream, d, n), words)
    assert np.array_equal(code.decode(stream, d, 5, first_bit=int(offs[n - 5])), words[n - 5:])  # rows decode on their own
    # (the two middle buckets of a symmetric law tie: the lengths depend on which of them an implementation's
    # masses make larger by 1e-9, so the oracle's construction is run on the same masses)
    assert np.max(np.abs(masses - o.bucket_masses(o.lloyd_max_codebook(d, bits)[0], d))) < 1e-8
    L = o.huffman_lengths(masses)
    buckets = o.unpack_planes(words, bits, d)
    assert int(offs[n]) == int(L[buckets].sum())
    per_coord = int(offs[n]) / (n * d)
    assert per_coord < bits
    if bits == 4:
        assert abs((1 - per_coord / bits) - 0.05) < 0.01


def test_recall_harness_agrees_with_the_oracle():
    d, n, nq, bits = 128, 3000, 60, 3
    got = R.recall_at_k(tq, torch, W, d, n, nq, bits, "prod", "gaussian")
    # the same experiment through the oracle
    Pi = o.rotation_from_gaussian(W.gaussian_matrix(d, 101))
    S = W.sketch_matrix(d, 201)
    c32, t32, _ = o.codebook_fp32(d, bits - 1)
    x = W.unit_gaussian_rows(n, d, 4)
    q = W.gaussian_queries(nq, d, 5, unit=True)
    r = o.quant_prod(x, Pi, S, c32, t32)
    est = o.score(q, o.dequant_prod(r["idx"], r["qjl"], r["gamma"], Pi, S, c32, r["norm"]))
    order = np.argsort(-est, axis=1, kind="stable")
    truth = np.argmax(q.astype(np.float64) @ x.astype(np.float64).T, axis=1)
    for k in R.KS:
        want = float(np.mean([truth[i] in order[i, :k] for i in range(nq)]))
        assert abs(got[f"1@{k}"] - want) <= 1.0 / nq + 1e-9, (k, got[f"1@{k}"], want)
    vals = [got[f"1@{k}"] for k in R.KS]
    assert all(a <= b for a, b in zip(vals, vals[1:]))
