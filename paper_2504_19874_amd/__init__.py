"""MI355X-native TurboQuant (arxiv 2504.19874): batched quantisation,
dequantisation and inner-product scoring as hand-written HIP kernels behind a
small C ABI (include/turboquant.h).  This package is the thin binding."""
from .api import (Params, TurboQuantError, tq_append, tq_attend, tq_attend_workspace_bytes, tq_build_codebook, tq_dequantize, tq_quantize_mse,
                  tq_quantize_prod, tq_score, tq_score_static, tq_score_static_scratch_bytes, tq_stage_pack, tq_stage_sign_pack, tq_stage_unpack,
                  tq_images_bytes, tq_workspace_bytes)
from .params import make_mixed_params, make_params, rotation_from_gaussian

__all__ = ["Params", "TurboQuantError", "tq_append", "tq_attend", "tq_attend_workspace_bytes", "tq_build_codebook", "tq_dequantize", "tq_quantize_mse",
           "tq_quantize_prod", "tq_score", "tq_score_static", "tq_score_static_scratch_bytes", "tq_stage_pack", "tq_stage_sign_pack", "tq_stage_unpack",
           "tq_images_bytes", "tq_workspace_bytes", "make_params", "make_mixed_params", "rotation_from_gaussian"]
