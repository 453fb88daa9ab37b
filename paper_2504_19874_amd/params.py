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
