"""Quality harness on synthetic data: recall 1@k of the nearest-neighbour
search of Sec. 4.4 and the distortions of Sec. 4.1 against Theorems 1-3.

    python -m paper_2504_19874_amd.recall --d 1536 --n 100000 --nq 1000 --bits 2 4 [--kind mse prod] [--data gaussian]
    python -m paper_2504_19874_amd.recall --distortion --d 1536 --n 20000 --bits 1 2 3 4
    python -m paper_2504_19874_amd.recall --entropy --d 1536 --n 20000 --bits 2 3 4

Recall 1@k (Sec. 4.4): the fraction of queries whose true maximum-inner-product
database vector is among the k best of the estimated scores.  The database is
quantised, scored and ranked by the library (tq_quantize_*, tq_score with
top-k); the ground truth is an exact fp32 brute force (a plain matrix product,
in chunks) and is not part of the method.  Inputs are the seeded cluster
mixture of workloads/ (unit-norm rows, queries from the same mixture), which
stands in for the embedding datasets of the paper: absolute recall values are
those of this synthetic set, not the paper's.

Distortion (Sec. 4.1, Fig. 3): D_mse = E||x - x~||^2 of unit vectors and
D_prod = E|<y,x> - est|^2 for unit-norm queries y, next to the upper bounds
of Theorems 1 and 2 and the lower bound of Theorem 3.  One JSON line per
setting.

Entropy (Sec. 3.1, the remark on entropy coding the indices): the empirical
entropy of the stored indices in bits per coordinate, i.e. what a prefix code
over the bucket probabilities could reach instead of b.  The library stores
plain b-bit indices, as the paper's own implementation does; this is the
measurement only.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

KS = (1, 2, 4, 8, 16, 32, 64)


def _params(tq, W, d, bits, kind, seed_pi=101, seed_s=201):
    prod = kind == "prod"
    S = W.sketch_matrix(d, seed_s) if prod else None
    return tq.make_params(d, bits - 1 if prod else bits, W.gaussian_matrix(d, seed_pi), S)


def _quantize(tq, torch, p, x, prod):
    n = x.shape[0]
    idx = torch.zeros((n, max(1, p.idx_words)), dtype=torch.int32, device="cuda")
    norm = torch.zeros(n, dtype=torch.float32, device="cuda")
    if prod:
        qjl = torch.zeros((n, p.qjl_words), dtype=torch.int32, device="cuda")
        gamma = torch.zeros(n, dtype=torch.float32, device="cuda")
        tq.tq_quantize_prod(p, x, idx, qjl, gamma, norm)
        return idx, qjl, gamma, norm
    tq.tq_quantize_mse(p, x, idx, norm)
    return idx, None, None, norm


def true_argmax(torch, q, x, chunk=65536):
    """Index of the largest exact inner product per query (ties: lowest index)."""
    best_v = torch.full((q.shape[0],), -float("inf"), device=q.device)
    best_i = torch.zeros((q.shape[0],), dtype=torch.int64, device=q.device)
    for s in range(0, x.shape[0], chunk):
        v, i = (q @ x[s:s + chunk].T).max(dim=1)
        take = v > best_v
        best_v = torch.where(take, v, best_v)
        best_i = torch.where(take, i + s, best_i)
    return best_i


def recall_at_k(tq, torch, W, d, n, nq, bits, kind, data="mixture", seed_x=4, seed_q=5):
    prod = kind == "prod"
    p = _params(tq, W, d, bits, kind).reserve(n, nq, max(KS))
    if data == "mixture":  # the cluster mixture of the ANN configurations: many near-equal candidates
        centers = W.mixture_centers(d, seed_x)
        x = torch.empty((n, d), dtype=torch.float32, device="cuda")
        for start, blk in W.mixture_rows(n, d, seed_x, seed_x):
            x[start:start + blk.shape[0]] = torch.from_numpy(blk).cuda()
        q = torch.from_numpy(W.mixture_chunk(0, nq, d, seed_q, centers)).cuda()
    else:  # isotropic unit vectors
        x = torch.from_numpy(W.unit_gaussian_rows(n, d, seed_x)).cuda()
        q = torch.from_numpy(W.gaussian_queries(nq, d, seed_q, unit=True)).cuda()
    idx, qjl, gamma, norm = _quantize(tq, torch, p, x, prod)
    ti = torch.zeros((nq, max(KS)), dtype=torch.int32, device="cuda")
    tq.tq_score(p, q, 1, nq, idx if p.idx_words else None, qjl, gamma, norm, n, None, max(KS), ti, None)
    truth = true_argmax(torch, q, x)
    hit = ti.to(torch.int64) == truth[:, None]
    return {f"1@{k}": float(hit[:, :k].any(dim=1).float().mean()) for k in KS}


def distortion(tq, torch, W, d, n, nq, bits, kind, seed_x=4, seed_q=5):
    prod = kind == "prod"
    p = _params(tq, W, d, bits, kind).reserve(n, nq, 0)
    x = torch.from_numpy(W.unit_gaussian_rows(n, d, seed_x)).cuda()
    q = torch.from_numpy(W.gaussian_queries(nq, d, seed_q, unit=True)).cuda()
    idx, qjl, gamma, norm = _quantize(tq, torch, p, x, prod)
    xt = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    tq.tq_dequantize(p, idx if p.idx_words else None, qjl, gamma, norm, xt)
    s = torch.zeros((nq, n), dtype=torch.float32, device="cuda")
    tq.tq_score(p, q, 1, nq, idx if p.idx_words else None, qjl, gamma, norm, n, s)
    exact = q.double() @ x.double().T
    err = s.double() - exact
    return {"D_mse": float(((x.double() - xt.double()) ** 2).sum(dim=1).mean()),
            "D_prod": float((err ** 2).mean()), "bias": float(err.mean()),
            # slope of the estimate against the truth: 1 for an unbiased estimator (Theorem 2),
            # below 1 for the MSE quantiser at low bit widths (Sec. 3.2)
            "slope": float((s.double() * exact).sum() / (exact * exact).sum()),
            "upper_mse": math.sqrt(3.0) * math.pi / 2.0 * 4.0 ** -bits,
            "upper_prod": math.sqrt(3.0) * math.pi ** 2 / d * 4.0 ** -bits,
            "lower_mse": 4.0 ** -bits, "lower_prod": 4.0 ** -bits / d}


def index_entropy(tq, torch, W, d, n, bits, seed_x=4):
    """Histogram of the indices the library stores for unit vectors -> entropy in bits per coordinate."""
    p = _params(tq, W, d, bits, "mse").reserve(n, 0, 0)
    x = torch.from_numpy(W.unit_gaussian_rows(n, d, seed_x)).cuda()
    idx, _, _, _ = _quantize(tq, torch, p, x, False)
    words = idx.view(n, d // 32, bits).to(torch.int64) & 0xFFFFFFFF  # [vector][group][plane]
    lanes = torch.arange(32, device="cuda")
    level = torch.zeros((n, d // 32, 32), dtype=torch.int64, device="cuda")
    for pl in range(bits):
        level |= ((words[:, :, pl, None] >> lanes) & 1) << pl
    freq = torch.bincount(level.reshape(-1), minlength=1 << bits).double() / level.numel()
    nz = freq[freq > 0]
    h = float(-(nz * torch.log2(nz)).sum())
    return {"entropy_bits": h, "saving": 1.0 - h / bits, "freq": [round(float(f), 5) for f in freq]}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--d", type=int, default=1536)
    ap.add_argument("--n", type=int, default=100000)
    ap.add_argument("--nq", type=int, default=1000)
    ap.add_argument("--bits", type=int, nargs="+", default=[2, 4])
    ap.add_argument("--kind", nargs="+", default=["mse", "prod"])
    ap.add_argument("--distortion", action="store_true")
    ap.add_argument("--entropy", action="store_true")
    ap.add_argument("--data", choices=["mixture", "gaussian"], default="mixture")
    args = ap.parse_args()

    import torch

    import paper_2504_19874_amd as tq
    import workloads as W

    if args.entropy:
        for bits in args.bits:
            out = {"d": args.d, "n": args.n, "bits": bits}
            out.update(index_entropy(tq, torch, W, args.d, args.n, bits))
            print(json.dumps(out), flush=True)
        return
    for kind in args.kind:
        for bits in args.bits:
            out = {"d": args.d, "n": args.n, "nq": args.nq, "bits": bits, "kind": kind}
            if args.distortion:
                out.update(distortion(tq, torch, W, args.d, args.n, args.nq, bits, kind))
            else:
                out["data"] = args.data
                out.update(recall_at_k(tq, torch, W, args.d, args.n, args.nq, bits, kind, args.data))
            print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
