"""tq_score_static (the entry point that allocates nothing: its scratch memory is a static device array)
against tq_score on the same codes, and both against the oracle, through the C ABI.  Two calls in a row,
the second with a smaller input, on each scoring route that uses scratch memory."""
import ctypes as C

import numpy as np
import pytest
import torch

import workloads as W
from oracle import turboquant_oracle as o
from tests import parity as P

pytestmark = pytest.mark.gpu

tq = pytest.importorskip("paper_2504_19874_amd")


def _codes(d, bits_mse, prod, n, seed):
    """Random valid codes (the scoring calls take any code) and their oracle dequantisation."""
    rng = np.random.default_rng([seed, d, n])
    Pi = o.rotation_from_gaussian(W.gaussian_matrix(d, 100))
    S = W.sketch_matrix(d, 200) if prod else None
    c32, t32, _ = o.codebook_fp32(d, bits_mse)
    idx = rng.integers(0, 1 << bits_mse, size=(n, d)).astype(np.int32)
    z = rng.integers(0, 2, size=(n, d)).astype(bool)
    gamma = rng.uniform(0.2, 0.6, size=n).astype(np.float32)
    norm = rng.uniform(0.5, 3.0, size=n).astype(np.float32)
    want = o.dequant_prod(idx, z, gamma, Pi, S, c32, norm) if prod else o.dequant_mse(idx, Pi, c32, norm)
    p = tq.Params(d, bits_mse, torch.from_numpy(Pi), None if S is None else torch.from_numpy(S), c32, t32)
    dev = lambda a: torch.as_tensor(np.ascontiguousarray(a)).cuda()
    t = dict(idx=dev(o.pack_planes(idx, bits_mse).view(np.int32)),
             qjl=dev(o.pack_signs(z).view(np.int32)) if prod else None,
             gamma=dev(gamma) if prod else None, norm=dev(norm))
    return p, t, want, norm


def _raw_call(fn, p, q, n_groups, qpg, t, n_per_group, scores, topk, ti, tv):
    ptr = lambda x: None if x is None else C.c_void_p(x.data_ptr())
    return fn(C.byref(p.c), ptr(q), q.stride(0), n_groups, qpg, ptr(t["idx"]), ptr(t["qjl"]), ptr(t["gamma"]),
              ptr(t["norm"]), n_per_group, ptr(scores), n_per_group if scores is None else scores.stride(0), topk,
              ptr(ti), ptr(tv), C.c_void_p(torch.cuda.current_stream().cuda_stream))


# (d, bits_mse, prod, n_groups, q_per_group, first n_per_group, second n_per_group, topk): the int8 route at
# d = 128 (digit images in scratch), the int8 route with a preparation kernel, the lane-per-key route and the
# many-query contraction (rotated queries in scratch), top-k without a score buffer (scores in scratch)
CASES = [(128, 2, True, 8, 4, 3000, 517, 0), (256, 3, False, 2, 8, 1500, 300, 0), (96, 2, True, 3, 5, 900, 130, 0),
         (128, 4, False, 1, 100, 2500, 700, 10), (160, 1, True, 1, 70, 1100, 256, 5)]


@pytest.mark.parametrize("d,bits_mse,prod,n_groups,qpg,n1,n2,topk", CASES)
def test_static_scratch_scoring_equals_tq_score(d, bits_mse, prod, n_groups, qpg, n1, n2, topk):
    from paper_2504_19874_amd import _lib
    lib = _lib.load()
    assert lib.tq_score_static_scratch_bytes() == 16 << 20
    nq = n_groups * qpg
    for n_per_group in (n1, n2):  # two calls in a row on the same array, the second smaller
        p, t, want, norm = _codes(d, bits_mse, prod, n_groups * n_per_group, 7)
        q_h = W.gaussian_queries(nq, d, 11, unit=False)
        q = torch.from_numpy(q_h).cuda()
        p.reserve(n_groups * n_per_group, nq, topk)
        ref = torch.zeros((nq, n_per_group), dtype=torch.float32, device="cuda")
        ref_ti = torch.zeros((nq, max(1, topk)), dtype=torch.int32, device="cuda")
        ref_tv = torch.zeros((nq, max(1, topk)), dtype=torch.float32, device="cuda")
        assert _raw_call(lib.tq_score, p, q, n_groups, qpg, t, n_per_group, ref, topk, ref_ti if topk else None,
                         ref_tv if topk else None) == 0
        # the new entry point never sees a workspace
        p.c.workspace, p.c.workspace_bytes = 0, 0
        got = torch.full((nq, n_per_group), float("nan"), dtype=torch.float32, device="cuda")
        got_ti = torch.full((nq, max(1, topk)), -7, dtype=torch.int32, device="cuda")
        got_tv = torch.full((nq, max(1, topk)), float("nan"), dtype=torch.float32, device="cuda")
        assert _raw_call(lib.tq_score_static, p, q, n_groups, qpg, t, n_per_group, got, topk,
                         got_ti if topk else None, got_tv if topk else None) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, ref)  # same kernels on the same inputs: identical bits
        for g in range(n_groups):
            rows = slice(g * qpg, (g + 1) * qpg)
            cols = slice(g * n_per_group, (g + 1) * n_per_group)
            P.check_close(got[rows].cpu().numpy(), o.score(q_h[rows], want[cols]),
                          np.linalg.norm(q_h[rows], axis=1)[:, None] * norm[cols][None, :], "score")
        if topk:
            assert torch.equal(got_ti, ref_ti) and torch.equal(got_tv, ref_tv)
            # and without a score buffer: the score matrix lives in the static array
            only_ti = torch.full_like(got_ti, -7)
            assert _raw_call(lib.tq_score_static, p, q, n_groups, qpg, t, n_per_group, None, topk, only_ti, None) == 0
            torch.cuda.synchronize()
            assert torch.equal(only_ti, ref_ti)


def test_static_scratch_rejects_what_does_not_fit():
    from paper_2504_19874_amd import _lib
    lib = _lib.load()
    p, t, _, _ = _codes(128, 2, False, 64, 3)
    p.c.workspace, p.c.workspace_bytes = 0, 0
    nq = 40000  # 2 x 40000 x 128 floats of rotated queries: more than 16 MiB
    q = torch.zeros((nq, 128), dtype=torch.float32, device="cuda")
    s = torch.zeros((nq, 64), dtype=torch.float32, device="cuda")
    assert _raw_call(lib.tq_score_static, p, q, 1, nq, t, 64, s, 0, None, None) == 4  # TQ_ERR_WORKSPACE
    # top-k without a score buffer on a route that keeps a score matrix in scratch memory (few queries per
    # code): 32 x 200000 floats do not fit
    ti = torch.zeros((32, 4), dtype=torch.int32, device="cuda")
    p2, t2, _, _ = _codes(128, 2, False, 200000, 4)
    p2.c.workspace, p2.c.workspace_bytes = 0, 0
    assert _raw_call(lib.tq_score_static, p2, q[:32], 1, 32, t2, 200000, None, 4, ti, None) == 4
    # the same request with many queries per code selects inside the scoring kernel and fits
    ti = torch.zeros((64, 4), dtype=torch.int32, device="cuda")
    assert _raw_call(lib.tq_score_static, p2, q[:64], 1, 64, t2, 200000, None, 4, ti, None) == 0
    torch.cuda.synchronize()
    assert torch.equal(ti.cpu(), torch.arange(4, dtype=torch.int32).repeat(64, 1))  # zero queries: all scores 0, ties by index
    assert lib.tq_status_string(4) == b"TQ_ERR_WORKSPACE"
