"""vlac: VLA-Cache sparse prefill on MI355X.  Thin ctypes binding over the C ABI
declared in include/vlac.h; every computation runs in libvlac.so's HIP kernels."""
from .binding import (VlacError, ModelCfg, LayerW, OPERAND_BF16, OPERAND_F16, OPERAND_F16_W8, lib, lib_path, use_library, status_string,
                      vlac_create, vlac_destroy, vlac_set_layer_weights, vlac_set_head_weights,
                      vlac_kv_cache_bytes, vlac_plan_many_rows_gemm, vlac_reset_stream, vlac_check, vlac_select_static, vlac_select_static_noalloc, vlac_embed_patches, vlac_quantize_e4m3,
                      vlac_layer_ratio, vlac_sparse_prefill, vlac_decode_action,
                      vlac_last_hip_error, vlac_profile_select, vlac_profile_read,
                      vlac_profile_read2, vlac_profile_bracket_cost)

__all__ = [n for n in dir() if n.startswith("vlac_")] + [
    "VlacError", "ModelCfg", "LayerW", "OPERAND_BF16", "OPERAND_F16", "OPERAND_F16_W8", "lib", "lib_path", "use_library", "status_string"]
