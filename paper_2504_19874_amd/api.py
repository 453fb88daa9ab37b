"""Thin Python binding of the C ABI in include/turboquant.h.

Argument marshalling only: every function takes torch tensors that already
live on the GPU (plus numpy arrays for the host-side codebook), passes their
addresses and the current HIP stream to the library, and raises on a non-zero
status.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes as C

import numpy as np
import torch

from . import _lib

TQ_F32, TQ_BF16 = 0, 1


class TurboQuantError(RuntimeError):
    pass


def _check(status: int, what: str):
    if status != 0:
        name = _lib.load().tq_status_string(status).decode()
        raise TurboQuantError(f"{what}: {name}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise TurboQuantError("expected a GPU tensor")
    if not t.is_contiguous():
        raise TurboQuantError("expected a contiguous tensor")
    return C.c_void_p(t.data_ptr())


def _ptr_rows(t):
    """A matrix whose row stride is passed separately: rows may be padded."""
    if t is None:
        return None
    if not t.is_cuda:
        raise TurboQuantError("expected a GPU tensor")
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise TurboQuantError("expected a matrix with contiguous rows")
    return C.c_void_p(t.data_ptr())


def _need(t, dtype, numel, what):
    """A code array must have the dtype the library writes and at least `numel` elements: the library only
    sees an address, so a short or mistyped tensor would be read or written past its end."""
    if t is None:
        return
    if t.dtype != dtype:
        raise TurboQuantError(f"{what}: expected {dtype}, got {t.dtype}")
    if t.numel() < numel:
        raise TurboQuantError(f"{what}: {t.numel()} elements where the call covers {numel}")


def _check_codes(p, rows, idx, qjl, gamma, norm):
    _need(idx, torch.int32, rows * p.idx_words, "idx")
    _need(qjl, torch.int32, rows * p.qjl_words, "qjl")
    _need(gamma, torch.float32, rows * p.scalars_per_vector, "gamma")
    _need(norm, torch.float32, rows * p.scalars_per_vector, "norm")


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def tq_build_codebook(d: int, bits: int):
    """-> (centroids float32[2^bits], bounds float32[2^bits-1], cost_per_coord)."""
    lib = _lib.load()
    c = np.zeros(1 << bits, dtype=np.float32)
    t = np.zeros(max(1, (1 << bits) - 1), dtype=np.float32)
    cost = C.c_double(0.0)
    _check(lib.tq_build_codebook(d, bits, c.ctypes.data_as(C.c_void_p), t.ctypes.data_as(C.c_void_p),
                                 C.byref(cost)), "tq_build_codebook")
    return c, t[: (1 << bits) - 1].copy(), cost.value


class Params:
    """Owns the tq_params struct and keeps every buffer it points to alive."""

    def __init__(self, d: int, bits_mse: int, Pi: torch.Tensor, S: torch.Tensor | None,
                 centroids: np.ndarray, bounds: np.ndarray, device="cuda", d_hi: int = 0, bits_mse_hi: int = 0,
                 centroids_hi: np.ndarray | None = None, bounds_hi: np.ndarray | None = None):
        """d_hi > 0: two instances over a split of the rotated coordinates (Sec. 4.3); then
        (bits_mse, centroids, bounds) belong to the d - d_hi coordinates of instance lo and the
        *_hi arguments to the first d_hi."""
        lib = _lib.load()
        self.d, self.bits_mse = int(d), int(bits_mse)
        self.device = torch.device(device)
        self.Pi = Pi.to(self.device, torch.float32).contiguous()
        self.S = None if S is None else S.to(self.device, torch.float32).contiguous()
        self.PiT = torch.empty_like(self.Pi)
        self.ST = None if S is None else torch.empty_like(self.S)
        self.SPiT = None if S is None else torch.empty_like(self.S)
        self.centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        self.bounds = np.ascontiguousarray(bounds, dtype=np.float32)
        if self.centroids.size != (1 << bits_mse) or self.bounds.size != (1 << bits_mse) - 1:
            raise TurboQuantError("codebook size does not match bits_mse")
        self._bounds_buf = self.bounds if self.bounds.size else np.zeros(1, dtype=np.float32)
        self.workspace = None
        self.c = _lib.TqParams()
        self.c.d, self.c.bits_mse = self.d, self.bits_mse
        self.c.Pi, self.c.PiT = self.Pi.data_ptr(), self.PiT.data_ptr()
        self.c.S = 0 if self.S is None else self.S.data_ptr()
        self.c.ST = 0 if self.ST is None else self.ST.data_ptr()
        self.c.SPiT = 0 if self.SPiT is None else self.SPiT.data_ptr()
        self.c.centroids = self.centroids.ctypes.data
        self.c.bounds = self._bounds_buf.ctypes.data
        self.c.workspace, self.c.workspace_bytes = 0, 0
        self.d_hi, self.bits_mse_hi = int(d_hi), int(bits_mse_hi)
        self.c.d_hi, self.c.bits_mse_hi, self.c.centroids_hi, self.c.bounds_hi = 0, 0, 0, 0
        self.c.flags = 0
        if self.d_hi:
            self.centroids_hi = np.ascontiguousarray(centroids_hi, dtype=np.float32)
            self.bounds_hi = np.ascontiguousarray(bounds_hi, dtype=np.float32)
            if self.centroids_hi.size != (1 << bits_mse_hi) or self.bounds_hi.size != (1 << bits_mse_hi) - 1:
                raise TurboQuantError("codebook size does not match bits_mse_hi")
            self._bounds_hi_buf = self.bounds_hi if self.bounds_hi.size else np.zeros(1, dtype=np.float32)
            self.c.d_hi, self.c.bits_mse_hi = self.d_hi, self.bits_mse_hi
            self.c.centroids_hi = self.centroids_hi.ctypes.data
            self.c.bounds_hi = self._bounds_hi_buf.ctypes.data
        _check(lib.tq_derive_params(self.d, _ptr(self.Pi), _ptr(self.S), _ptr(self.PiT), _ptr(self.ST),
                                    _ptr(self.SPiT), _stream()), "tq_derive_params")
        self.c.images, self.images = 0, None
        self.build_images()

    def build_images(self):
        """The matrices in the form the large-batch d = 128 kernels keep on chip (tq_build_images); a no-op at
        other dimensions.  `drop_images` goes back to splitting them in every launch (same results)."""
        need = int(_lib.load().tq_images_bytes(self.d))
        if need:
            self.images = torch.empty(need, dtype=torch.uint8, device=self.device)
            _check(_lib.load().tq_build_images(C.byref(self.c), _ptr(self.images), _stream()), "tq_build_images")
            self.c.images = self.images.data_ptr()
        return self

    def drop_images(self):
        self.c.images, self.images = 0, None
        return self

    def reserve(self, n: int, nq: int = 0, topk: int = 0):
        """Size the device workspace for calls with up to n vectors / nq queries."""
        return self.reserve_bytes(tq_workspace_bytes(self, n, nq, topk))

    def reserve_bytes(self, need: int):
        """Make the device workspace at least `need` bytes."""
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)
            self.c.workspace = self.workspace.data_ptr()
            self.c.workspace_bytes = self.workspace.numel()
        return self

    def reserve_score(self, n_groups: int, q_per_group: int, n_per_group: int, prod: bool, scores_given: bool,
                      topk: int = 0):
        """Size the workspace for exactly one kind of tq_score call (tq_score_workspace_bytes)."""
        need = int(_lib.load().tq_score_workspace_bytes(C.byref(self.c), n_groups, q_per_group, n_per_group, int(prod),
                                                        int(scores_given), topk))
        if need == 0:
            raise TurboQuantError("tq_score_workspace_bytes: invalid arguments")
        return self.reserve_bytes(need)

    @property
    def fp32_mfma(self) -> bool:
        """TQ_FLAG_FP32_MFMA of the struct: every contraction on the fp32 matrix instructions."""
        return bool(self.c.flags & _lib.TQ_FLAG_FP32_MFMA)

    @fp32_mfma.setter
    def fp32_mfma(self, on: bool):
        self.c.flags = (self.c.flags | _lib.TQ_FLAG_FP32_MFMA) if on else (self.c.flags & ~_lib.TQ_FLAG_FP32_MFMA)

    @property
    def idx_words(self) -> int:
        return (self.d_hi // 32) * self.bits_mse_hi + ((self.d - self.d_hi) // 32) * self.bits_mse

    @property
    def scalars_per_vector(self) -> int:
        """Floats per vector in the gamma and norm arrays: one per instance."""
        return 2 if self.d_hi else 1

    @property
    def qjl_words(self) -> int:
        return self.d // 32


def tq_images_bytes(d: int) -> int:
    return int(_lib.load().tq_images_bytes(d))


def tq_workspace_bytes(p: Params, n: int, nq: int, topk: int) -> int:
    return int(_lib.load().tq_workspace_bytes(C.byref(p.c), n, nq, topk))


def _dtype_of(x: torch.Tensor) -> int:
    if x.dtype == torch.float32:
        return TQ_F32
    if x.dtype == torch.bfloat16:
        return TQ_BF16
    raise TurboQuantError(f"unsupported input dtype {x.dtype}")


def tq_quantize_mse(p: Params, x: torch.Tensor, idx: torch.Tensor, norm: torch.Tensor | None):
    n = x.shape[0]
    _check_codes(p, n, idx, None, None, norm)
    _check(_lib.load().tq_quantize_mse(C.byref(p.c), _ptr_rows(x), _dtype_of(x), n, x.stride(0) if n else p.d,
                                       _ptr(idx), _ptr(norm), _stream()), "tq_quantize_mse")


def tq_quantize_prod(p: Params, x: torch.Tensor, idx: torch.Tensor, qjl: torch.Tensor,
                     gamma: torch.Tensor, norm: torch.Tensor | None):
    n = x.shape[0]
    _check_codes(p, n, idx, qjl, gamma, norm)
    _check(_lib.load().tq_quantize_prod(C.byref(p.c), _ptr_rows(x), _dtype_of(x), n, x.stride(0) if n else p.d,
                                        _ptr(idx), _ptr(qjl), _ptr(gamma), _ptr(norm), _stream()),
           "tq_quantize_prod")


def tq_dequantize(p: Params, idx, qjl, gamma, norm, x_out: torch.Tensor):
    n = x_out.shape[0]
    _check_codes(p, n, idx, qjl, gamma, norm)
    _need(x_out, torch.float32, 0, "x_out")
    _check(_lib.load().tq_dequantize(C.byref(p.c), _ptr(idx), _ptr(qjl), _ptr(gamma), _ptr(norm), n,
                                     _ptr_rows(x_out), x_out.stride(0) if n else p.d, _stream()), "tq_dequantize")


def _check_score_args(p, q, n_groups, q_per_group, idx, qjl, gamma, norm, n_per_group, scores, topk, topk_idx, topk_val):
    nq = n_groups * q_per_group
    _check_codes(p, n_groups * n_per_group, idx, qjl, gamma, norm)
    _need(q, torch.float32, 0, "q")
    if q.shape[0] < nq:
        raise TurboQuantError(f"q: {q.shape[0]} rows for {nq} queries")
    if scores is not None:
        _need(scores, torch.float32, 0, "scores")
        if scores.shape[0] < nq or scores.shape[1] < n_per_group:
            raise TurboQuantError(f"scores: {tuple(scores.shape)} where the call writes {nq} x {n_per_group}")
    _need(topk_idx, torch.int32, nq * topk, "topk_idx")
    _need(topk_val, torch.float32, nq * topk, "topk_val")


def tq_score(p: Params, q: torch.Tensor, n_groups: int, q_per_group: int, idx, qjl, gamma, norm,
             n_per_group: int, scores: torch.Tensor | None, topk: int = 0,
             topk_idx: torch.Tensor | None = None, topk_val: torch.Tensor | None = None):
    lds = scores.stride(0) if scores is not None and scores.shape[0] else n_per_group
    _check_score_args(p, q, n_groups, q_per_group, idx, qjl, gamma, norm, n_per_group, scores, topk, topk_idx, topk_val)
    _check(_lib.load().tq_score(C.byref(p.c), _ptr_rows(q), q.stride(0) if q.shape[0] else p.d, n_groups,
                                q_per_group, _ptr(idx), _ptr(qjl), _ptr(gamma), _ptr(norm), n_per_group,
                                _ptr_rows(scores), lds, topk, _ptr(topk_idx), _ptr(topk_val), _stream()),
           "tq_score")


def tq_score_static(p: Params, q: torch.Tensor, n_groups: int, q_per_group: int, idx, qjl, gamma, norm,
                    n_per_group: int, scores: torch.Tensor | None, topk: int = 0,
                    topk_idx: torch.Tensor | None = None, topk_val: torch.Tensor | None = None):
    """tq_score on the library's static scratch array: p's workspace is not used and nothing is allocated."""
    lds = scores.stride(0) if scores is not None and scores.shape[0] else n_per_group
    _check_score_args(p, q, n_groups, q_per_group, idx, qjl, gamma, norm, n_per_group, scores, topk, topk_idx, topk_val)
    _check(_lib.load().tq_score_static(C.byref(p.c), _ptr_rows(q), q.stride(0) if q.shape[0] else p.d, n_groups,
                                       q_per_group, _ptr(idx), _ptr(qjl), _ptr(gamma), _ptr(norm), n_per_group,
                                       _ptr_rows(scores), lds, topk, _ptr(topk_idx), _ptr(topk_val), _stream()),
           "tq_score_static")


def tq_score_static_scratch_bytes() -> int:
    return int(_lib.load().tq_score_static_scratch_bytes())


def tq_attend_workspace_bytes(pk: Params, pv: Params, n_groups: int, q_per_group: int, n_per_group: int) -> int:
    return int(_lib.load().tq_attend_workspace_bytes(C.byref(pk.c), C.byref(pv.c), n_groups, q_per_group,
                                                     n_per_group))


def tq_append(p: Params, x: torch.Tensor, idx, qjl, gamma, norm, first_row: int, row_step: int):
    """Quantise the rows of x into code rows first_row + i * row_step of a cache (qjl None: the MSE quantiser)."""
    n = x.shape[0]
    if n:
        _check_codes(p, first_row + (n - 1) * row_step + 1, idx, qjl, gamma, norm)
    _check(_lib.load().tq_append(C.byref(p.c), _ptr_rows(x), _dtype_of(x), n, x.stride(0) if n else p.d, _ptr(idx),
                                 _ptr(qjl), _ptr(gamma), _ptr(norm), first_row, row_step, _stream()), "tq_append")


def tq_attend(pk: Params, pv: Params, q: torch.Tensor, n_groups: int, q_per_group: int, k_codes, v_codes,
              n_per_group: int, scale: float, out: torch.Tensor, group_stride: int | None = None):
    """k_codes, v_codes: (idx, qjl, gamma, norm) tensors, None where the quantiser has no such output.
    group_stride: token slots per group when the cache holds more than n_per_group (tq_attend_cache).
    Sizes pk's workspace for the call when it is too small."""
    need = tq_attend_workspace_bytes(pk, pv, n_groups, q_per_group, n_per_group)
    if pk.workspace is None or pk.workspace.numel() < need:
        pk.workspace = torch.empty(need, dtype=torch.uint8, device=pk.device)
        pk.c.workspace = pk.workspace.data_ptr()
        pk.c.workspace_bytes = pk.workspace.numel()
    if group_stride is not None:
        _check(_lib.load().tq_attend_cache(C.byref(pk.c), C.byref(pv.c), _ptr_rows(q), q.stride(0) if q.shape[0] else pk.d,
                                           n_groups, q_per_group, *[_ptr(t) for t in k_codes],
                                           *[_ptr(t) for t in v_codes], n_per_group, group_stride, C.c_float(scale),
                                           _ptr_rows(out), out.stride(0) if out.shape[0] else pv.d, _stream()),
               "tq_attend_cache")
        return
    _check(_lib.load().tq_attend(C.byref(pk.c), C.byref(pv.c), _ptr_rows(q), q.stride(0) if q.shape[0] else pk.d,
                                 n_groups, q_per_group, *[_ptr(t) for t in k_codes], *[_ptr(t) for t in v_codes],
                                 n_per_group, C.c_float(scale), _ptr_rows(out), out.stride(0) if out.shape[0] else pv.d,
                                 _stream()), "tq_attend")


def tq_stage_pack(p: Params, y: torch.Tensor, idx: torch.Tensor):
    _check(_lib.load().tq_stage_pack(C.byref(p.c), _ptr(y), y.shape[0], _ptr(idx), _stream()), "tq_stage_pack")


def tq_stage_sign_pack(d: int, u: torch.Tensor, qjl: torch.Tensor):
    _check(_lib.load().tq_stage_sign_pack(d, _ptr(u), u.shape[0], _ptr(qjl), _stream()), "tq_stage_sign_pack")


def tq_stage_unpack(p: Params, idx: torch.Tensor, y_tilde: torch.Tensor):
    _check(_lib.load().tq_stage_unpack(C.byref(p.c), _ptr(idx), y_tilde.shape[0], _ptr(y_tilde), _stream()),
           "tq_stage_unpack")
