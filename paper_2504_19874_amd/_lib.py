"""ctypes loader for libturboquant.so.  Fails loudly when the library has not
been built: there is no fallback path."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libturboquant.so")


class TqParams(C.Structure):
    _fields_ = [
        ("d", C.c_int32),
        ("bits_mse", C.c_int32),
        ("Pi", C.c_void_p),
        ("PiT", C.c_void_p),
        ("S", C.c_void_p),
        ("ST", C.c_void_p),
        ("SPiT", C.c_void_p),
        ("centroids", C.c_void_p),
        ("bounds", C.c_void_p),
        ("workspace", C.c_void_p),
        ("workspace_bytes", C.c_size_t),
        ("d_hi", C.c_int32),
        ("bits_mse_hi", C.c_int32),
        ("centroids_hi", C.c_void_p),
        ("bounds_hi", C.c_void_p),
        ("flags", C.c_uint32),
        ("images", C.c_void_p),
    ]

TQ_FLAG_FP32_MFMA = 1


_P = C.POINTER(TqParams)
_vp, _i32, _i64 = C.c_void_p, C.c_int32, C.c_int64

# name -> (restype, argtypes); mirrors include/turboquant.h
SIGNATURES = {
    "tq_status_string": (C.c_char_p, [C.c_int]),
    "tq_build_codebook": (C.c_int, [_i32, _i32, _vp, _vp, C.POINTER(C.c_double)]),
    "tq_bucket_masses": (C.c_int, [_i32, _i32, _vp, _vp]),
    "tq_images_bytes": (C.c_size_t, [_i32]),
    "tq_build_images": (C.c_int, [_P, _vp, _vp]),
    "tq_prefix_code_build": (C.c_int, [_i32, _vp, _vp, _vp, C.POINTER(C.c_double)]),
    "tq_entropy_encode": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _i64, _vp, C.c_size_t, C.POINTER(C.c_size_t), _vp]),
    "tq_entropy_decode": (C.c_int, [_i32, _i32, _vp, _vp, C.c_size_t, C.c_uint64, _i64, _vp]),
    "tq_build_rotation": (C.c_int, [_i32, _vp, _vp]),
    "tq_compose_split": (C.c_int, [_i32, _i32, _vp, _vp, _vp, _vp]),
    "tq_derive_params": (C.c_int, [_i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "tq_workspace_bytes": (C.c_size_t, [_P, _i64, _i64, _i32]),
    "tq_quantize_mse": (C.c_int, [_P, _vp, C.c_int, _i64, _i64, _vp, _vp, _vp]),
    "tq_quantize_prod": (C.c_int, [_P, _vp, C.c_int, _i64, _i64, _vp, _vp, _vp, _vp, _vp]),
    "tq_dequantize": (C.c_int, [_P, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "tq_score": (C.c_int, [_P, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i32, _vp, _vp, _vp]),
    "tq_score_workspace_bytes": (C.c_size_t, [_P, _i32, _i32, _i64, _i32, _i32, _i32]),
    "tq_score_static_scratch_bytes": (C.c_size_t, []),
    "tq_score_static": (C.c_int, [_P, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _i32, _vp, _vp, _vp]),
    "tq_attend_workspace_bytes": (C.c_size_t, [_P, _P, _i32, _i32, _i64]),
    "tq_attend": (C.c_int, [_P, _P, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, C.c_float, _vp,
                            _i64, _vp]),
    "tq_attend_cache": (C.c_int, [_P, _P, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64,
                                  C.c_float, _vp, _i64, _vp]),
    "tq_append": (C.c_int, [_P, _vp, C.c_int, _i64, _i64, _vp, _vp, _vp, _vp, _i64, _i64, _vp]),
    "tq_stage_pack": (C.c_int, [_P, _vp, _i64, _vp, _vp]),
    "tq_stage_sign_pack": (C.c_int, [_i32, _vp, _i64, _vp, _vp]),
    "tq_stage_unpack": (C.c_int, [_P, _vp, _i64, _vp, _vp]),
}

_lib = None


def load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2504_19874_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib
