"""Binding of the host-side entropy codec for stored indices (Sec. 3.1,
entropy-coding paragraph).  numpy arrays in host memory; marshalling only."""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import _lib
from .api import TurboQuantError, _check


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def bucket_masses(d: int, bits: int, centroids) -> np.ndarray:
    """p_l of the codebook's cells (tq_bucket_masses)."""
    c = np.ascontiguousarray(centroids, dtype=np.float32)
    if c.size != 1 << bits:
        raise TurboQuantError("codebook size does not match bits")
    p = np.zeros(1 << bits, dtype=np.float64)
    _check(_lib.load().tq_bucket_masses(d, bits, _p(c), _p(p)), "tq_bucket_masses")
    return p


class PrefixCode:
    """Optimal prefix code for index probabilities p (tq_prefix_code_build)."""

    def __init__(self, p):
        p = np.ascontiguousarray(p, dtype=np.float64)
        self.K = p.size
        self.bits = int(self.K).bit_length() - 1
        if 1 << self.bits != self.K:
            raise TurboQuantError("the number of indices must be a power of two")
        self.lengths = np.zeros(self.K, dtype=np.uint8)
        self.codewords = np.zeros(self.K, dtype=np.uint32)
        mean = C.c_double(0.0)
        _check(_lib.load().tq_prefix_code_build(self.K, _p(p), _p(self.lengths), _p(self.codewords), C.byref(mean)),
               "tq_prefix_code_build")
        self.mean_bits = mean.value

    def encode(self, idx_words: np.ndarray, d: int):
        """Packed index words [n, bits*d/32] -> (stream bytes, bit offset of every vector and of the end)."""
        w = np.ascontiguousarray(idx_words, dtype=np.uint32)
        n = w.shape[0]
        if w.ndim != 2 or w.shape[1] != self.bits * d // 32:
            raise TurboQuantError("idx_words does not have bits*d/32 words per vector")
        out = np.zeros(max(1, n * d * 4), dtype=np.uint8)
        used = C.c_size_t(0)
        offs = np.zeros(n + 1, dtype=np.uint64)
        _check(_lib.load().tq_entropy_encode(d, self.bits, _p(self.lengths), _p(self.codewords), _p(w), n, _p(out),
                                             out.size, C.byref(used), _p(offs)), "tq_entropy_encode")
        return out[:used.value].copy(), offs

    def decode(self, stream: np.ndarray, d: int, n: int, first_bit: int = 0) -> np.ndarray:
        s = np.ascontiguousarray(stream, dtype=np.uint8)
        out = np.zeros((n, self.bits * d // 32), dtype=np.uint32)
        _check(_lib.load().tq_entropy_decode(d, self.bits, _p(self.lengths), _p(s), s.size, first_bit, n, _p(out)),
               "tq_entropy_decode")
        return out
