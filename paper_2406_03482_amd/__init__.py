"""MI355X-native QJL key-cache hot path (arXiv 2406.03482).

The computation lives in `libqjl.so` (hand-written HIP for gfx950, C ABI in
`include/qjl.h`); this package is the thin ctypes binding around it plus the
seeded synthetic-input generators.  There is no CPU fallback: every function
raises if the library has not been built (`python -m paper_2406_03482_amd.build`).
"""
from .binding import (QJLShape, QJLError, lib, lib_path, qjl_make_sketch, qjl_make_sketch_orthogonal, qjl_quantize_keys,
                      qjl_project_query, qjl_scores, qjl_decode_workspace_bytes,
                      qjl_decode_attention, qjl_decode_plan, qjl_decode_attention_noalloc, qjl_select_outliers, qjl_make_dual_sketch,
                      qjl_quantize_keys_dual, qjl_decode_dual_workspace_bytes,
                      qjl_decode_attention_dual, qjl_quantize_values, qjl_decode_attention_vq, qjl_append_keys, qjl_decode_step,
                      qjl_decode_attention_dual_vq, qjl_generation_step,
                      QJL_F32, QJL_F16, QJL_BF16)

__all__ = ["QJLShape", "QJLError", "lib", "lib_path", "qjl_make_sketch", "qjl_make_sketch_orthogonal", "qjl_quantize_keys",
           "qjl_project_query", "qjl_scores", "qjl_decode_workspace_bytes",
           "qjl_decode_attention", "qjl_decode_plan", "qjl_decode_attention_noalloc", "qjl_select_outliers", "qjl_make_dual_sketch",
           "qjl_quantize_keys_dual", "qjl_decode_dual_workspace_bytes", "qjl_decode_attention_dual",
           "qjl_quantize_values", "qjl_decode_attention_vq", "qjl_append_keys", "qjl_decode_step",
           "qjl_decode_attention_dual_vq", "qjl_generation_step", "QJL_F32", "QJL_F16", "QJL_BF16"]
