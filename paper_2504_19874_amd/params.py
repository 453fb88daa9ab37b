"""Setup helpers for the global parameters of Alg. 1 / Alg. 2 (host side,
run once per (d, b), off the timed path)."""
from __future__ import annotations

import numpy as np
import torch

from . import api


def rotation_from_gaussian(G) -> torch.Tensor:
    """Random rotation of Sec. 3.1: the orthogonal factor of a QR decomposition
    of a matrix with i.i.d. normal entries.  Column j of the factor is flipped
    where R[j, j] is negative, which fixes the factor uniquely (R gets a
    positive diagonal) and makes it Haar distributed.  fp64 on the host,
    returned as fp32."""
    g = torch.as_tensor(np.asarray(G), dtype=torch.float64)
    qf, rf = torch.linalg.qr(g, mode="reduced")
    flip = torch.where(torch.diagonal(rf) < 0, -1.0, 1.0).to(torch.float64)
    return (qf * flip.unsqueeze(0)).to(torch.float32)


def make_params(d: int, bits_mse: int, gaussian_for_pi, S=None, device="cuda") -> api.Params:
    """Codebook from the library's own builder, Pi from the given Gaussian
    matrix, S as given (None for the MSE variant)."""
    c, t, _ = api.tq_build_codebook(d, bits_mse)
    Pi = rotation_from_gaussian(gaussian_for_pi)
    S_t = None if S is None else torch.as_tensor(np.asarray(S), dtype=torch.float32)
    return api.Params(d, bits_mse, Pi, S_t, c, t, device=device)


def make_mixed_params(d: int, hi_channels, bits_mse_hi: int, bits_mse_lo: int, gaussian_hi, gaussian_lo,
                      S_hi=None, S_lo=None, device="cuda") -> api.Params:
    """Two independent instances over a channel split (Sec. 4.3): the channels listed in
    hi_channels (outliers) form an instance of dimension len(hi_channels) with bits_mse_hi bits,
    the others one of dimension d - len(hi_channels) with bits_mse_lo bits.  Returned as one set
    of d x d parameters: Pi = blockdiag(Pi_hi, Pi_lo) P and S = blockdiag(S_hi, S_lo) P with P the
    permutation that lists the hi channels first (both in ascending order), so the kernels see x
    in its original channel order and rotated coordinates [0, d_hi) belong to instance hi."""
    hi = np.sort(np.asarray(hi_channels, dtype=np.int64))
    lo = np.setdiff1d(np.arange(d), hi)
    d_hi, d_lo = hi.size, lo.size
    order = np.concatenate([hi, lo])

    def blockdiag(a, b):
        m = torch.zeros((d, d), dtype=torch.float32)
        m[:d_hi, :d_hi] = torch.as_tensor(np.asarray(a), dtype=torch.float32)
        m[d_hi:, d_hi:] = torch.as_tensor(np.asarray(b), dtype=torch.float32)
        out = torch.zeros_like(m)
        out[:, order] = m  # column c of the block matrix acts on channel order[c]
        return out

    Pi = blockdiag(rotation_from_gaussian(gaussian_hi), rotation_from_gaussian(gaussian_lo))
    S = None if S_hi is None else blockdiag(S_hi, S_lo)
    c_hi, t_hi, _ = api.tq_build_codebook(d_hi, bits_mse_hi)
    c_lo, t_lo, _ = api.tq_build_codebook(d_lo, bits_mse_lo)
    return api.Params(d, bits_mse_lo, Pi, S, c_lo, t_lo, device=device, d_hi=d_hi, bits_mse_hi=bits_mse_hi,
                      centroids_hi=c_hi, bounds_hi=t_hi)
