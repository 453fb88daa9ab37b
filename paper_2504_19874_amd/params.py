"""Setup helpers for the global parameters of Alg. 1 / Alg. 2 (run once per
(d, b), off the timed path).  The arithmetic is the library's: the rotation
comes from tq_build_rotation, the codebook from tq_build_codebook, the
two-instance matrices from tq_compose_split; this module only passes arrays."""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import _lib, api


def rotation_from_gaussian(G) -> torch.Tensor:
    """Random rotation of Sec. 3.1 from a d x d matrix of N(0,1) draws (tq_build_rotation); fp32."""
    g = np.ascontiguousarray(np.asarray(G), dtype=np.float64)
    if g.ndim != 2 or g.shape[0] != g.shape[1]:
        raise api.TurboQuantError("expected a square matrix")
    out = np.empty(g.shape, dtype=np.float32)
    api._check(_lib.load().tq_build_rotation(g.shape[0], g.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p)),
               "tq_build_rotation")
    return torch.from_numpy(out)


def make_params(d: int, bits_mse: int, gaussian_for_pi, S=None, device="cuda") -> api.Params:
    """Codebook from the library's own builder, Pi from the given Gaussian
    matrix, S as given (None for the MSE variant)."""
    c, t, _ = api.tq_build_codebook(d, bits_mse)
    Pi = rotation_from_gaussian(gaussian_for_pi)
    S_t = None if S is None else torch.as_tensor(np.asarray(S), dtype=torch.float32)
    return api.Params(d, bits_mse, Pi, S_t, c, t, device=device)


def compose_split(d: int, hi_channels, block_hi, block_lo) -> torch.Tensor:
    """blockdiag(block_hi, block_lo) P with P listing hi_channels first (tq_compose_split)."""
    hi = np.ascontiguousarray(np.sort(np.asarray(hi_channels)), dtype=np.int32)
    a = np.ascontiguousarray(np.asarray(block_hi), dtype=np.float32)
    b = np.ascontiguousarray(np.asarray(block_lo), dtype=np.float32)
    if a.shape != (hi.size, hi.size) or b.shape != (d - hi.size, d - hi.size):
        raise api.TurboQuantError("block shapes do not match the channel split")
    out = np.empty((d, d), dtype=np.float32)
    api._check(_lib.load().tq_compose_split(d, hi.size, hi.ctypes.data_as(C.c_void_p), a.ctypes.data_as(C.c_void_p),
                                            b.ctypes.data_as(C.c_void_p), out.ctypes.data_as(C.c_void_p)),
               "tq_compose_split")
    return torch.from_numpy(out)


def make_mixed_params(d: int, hi_channels, bits_mse_hi: int, bits_mse_lo: int, gaussian_hi, gaussian_lo,
                      S_hi=None, S_lo=None, device="cuda") -> api.Params:
    """Two independent instances over a channel split (Sec. 4.3): the channels listed in
    hi_channels (outliers) form an instance of dimension len(hi_channels) with bits_mse_hi bits,
    the others one of dimension d - len(hi_channels) with bits_mse_lo bits.  Returned as one set
    of d x d parameters: Pi = blockdiag(Pi_hi, Pi_lo) P and S = blockdiag(S_hi, S_lo) P with P the
    permutation that lists the hi channels first (both in ascending order), so the kernels see x
    in its original channel order and rotated coordinates [0, d_hi) belong to instance hi."""
    d_hi = len(np.asarray(hi_channels))
    Pi = compose_split(d, hi_channels, rotation_from_gaussian(gaussian_hi).numpy(),
                       rotation_from_gaussian(gaussian_lo).numpy())
    S = None if S_hi is None else compose_split(d, hi_channels, S_hi, S_lo)
    c_hi, t_hi, _ = api.tq_build_codebook(d_hi, bits_mse_hi)
    c_lo, t_lo, _ = api.tq_build_codebook(d - d_hi, bits_mse_lo)
    return api.Params(d, bits_mse_lo, Pi, S, c_lo, t_lo, device=device, d_hi=d_hi, bits_mse_hi=bits_mse_hi,
                      centroids_hi=c_hi, bounds_hi=t_hi)
