"""ctypes binding of libvlac.so: argument marshalling only.

Pointer arguments may be torch tensors (their data_ptr() is passed; device,
dtype and contiguity are checked here), raw integer addresses, or None.
Functions raise VlacError on a negative status unless called with check=False,
in which case they return the status."""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

VLAC_OK, VLAC_E_NULL, VLAC_E_SHAPE, VLAC_E_RANGE, VLAC_E_STATE, VLAC_E_HIP, VLAC_E_NOMEM = (
    0, -1, -2, -3, -4, -5, -6)


class VlacError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, status_string(status), status))


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads",
                                         "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_base", C.c_float),
        ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("operand_dtype", C.c_int32)]


OPERAND_BF16, OPERAND_F16, OPERAND_F16_W8 = 0, 1, 2


class LayerW(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wqkv", "wo", "w_gate_up", "w_down", "g_attn", "g_ffn")]


_PATH = os.path.join(_HERE, "libvlac.so")
_LOADED = {}


def lib_path():
    return _PATH


def use_library(path=None):
    """Switches every later call of this binding to another build of the library (None: the
    product build, libvlac.so).  For the test that compares libvlac_safe.so, the build whose
    hand-placed waits are replaced by full waits, with the product build.  A context belongs
    to the library that created it: destroy it before switching."""
    global _LIB, _PATH
    if _LIB is not None:
        _LOADED[_PATH] = _LIB
    _PATH = path or os.path.join(_HERE, "libvlac.so")
    _LIB = _LOADED.get(_PATH)


def lib():
    """Loads libvlac.so (built by build.py); there is no fallback path."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError("libvlac.so is not built: run `python -m paper_2502_02175_amd.build` "
                              "(or __graft_entry__.build()); vlac has no CPU fallback")
        L = C.CDLL(path)
        vp, i32, f32 = C.c_void_p, C.c_int, C.c_float
        L.vlac_status_string.restype = C.c_char_p
        L.vlac_status_string.argtypes = [i32]
        L.vlac_plan_many_rows_gemm.restype = C.c_int
        L.vlac_plan_many_rows_gemm.argtypes = [C.c_int] * 4 + [C.POINTER(C.c_int)] * 3
        L.vlac_kv_cache_bytes.restype = C.c_size_t
        L.vlac_kv_cache_bytes.argtypes = [C.POINTER(ModelCfg)]
        L.vlac_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(vp)]
        L.vlac_destroy.argtypes = [vp]
        L.vlac_last_hip_error.argtypes = [vp]
        L.vlac_set_layer_weights.argtypes = [vp, i32, C.POINTER(LayerW), vp]
        L.vlac_set_head_weights.argtypes = [vp, vp, vp, vp, vp]
        L.vlac_reset_stream.argtypes = [vp, i32, vp, vp]
        L.vlac_check.argtypes = [vp, vp]
        L.vlac_profile_select.argtypes = [vp, i32]
        L.vlac_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
        L.vlac_profile_read2.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i32)]
        L.vlac_profile_bracket_cost.argtypes = [vp, vp, C.POINTER(C.c_double)]
        L.vlac_select_static.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, f32,
                                         vp, vp, vp, vp, i32, vp]
        L.vlac_select_static_noalloc.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, i32, vp, f32,
                                                 vp, vp, vp, vp, i32, vp]
        L.vlac_quantize_e4m3.argtypes = [vp, i32, i32, vp, vp, vp]
        L.vlac_embed_patches.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, i32, vp]
        L.vlac_layer_ratio.argtypes = [vp, vp, i32, i32, f32, vp, vp, vp, vp]
        L.vlac_sparse_prefill.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
        L.vlac_decode_action.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
        for name in ("vlac_create", "vlac_destroy", "vlac_last_hip_error", "vlac_set_layer_weights",
                     "vlac_set_head_weights", "vlac_reset_stream", "vlac_check",
                     "vlac_profile_select", "vlac_profile_read", "vlac_profile_read2",
                     "vlac_profile_bracket_cost",
                     "vlac_select_static", "vlac_select_static_noalloc", "vlac_embed_patches", "vlac_quantize_e4m3", "vlac_layer_ratio", "vlac_sparse_prefill",
                     "vlac_decode_action"):
            getattr(L, name).restype = i32
        _LIB = L
    return _LIB


def status_string(status):
    return lib().vlac_status_string(int(status)).decode()


def _ptr(x, dtype=None, name="argument"):
    """Device pointer of a torch tensor / raw address / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    import torch
    if not isinstance(x, torch.Tensor):
        raise TypeError("%s: expected a torch tensor, an address or None" % name)
    if not x.is_cuda:
        raise ValueError("%s must live in GPU memory" % name)
    if not x.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and x.dtype != dtype:
        raise TypeError("%s: dtype %s, expected %s" % (name, x.dtype, dtype))
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else 0
    return getattr(stream, "cuda_stream", stream)


def _ret(status, where, check):
    if check and status != VLAC_OK:
        raise VlacError(status, where)
    return status


def _cfg(cfg, max_batch=None, max_seq=None):
    if isinstance(cfg, ModelCfg):
        return cfg
    return ModelCfg(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                    cfg.d_ffn, cfg.vocab, cfg.rms_eps, cfg.rope_base, max_batch, max_seq)


def vlac_plan_many_rows_gemm(out_features, k, rows, max_splits=1):
    """-> (rows per work item, K parts, work items); no GPU needed."""
    tf, ks, wi = C.c_int(), C.c_int(), C.c_int()
    st = lib().vlac_plan_many_rows_gemm(out_features, k, rows, max_splits, C.byref(tf), C.byref(ks), C.byref(wi))
    if st != 0:
        raise VlacError(st, "vlac_plan_many_rows_gemm")
    return tf.value, ks.value, wi.value


def vlac_kv_cache_bytes(cfg):
    return int(lib().vlac_kv_cache_bytes(C.byref(cfg)))


def vlac_create(cfg, check=True):
    """Returns the context handle (an integer address)."""
    out = C.c_void_p()
    st = lib().vlac_create(C.byref(cfg) if cfg is not None else None, C.byref(out))
    _ret(st, "vlac_create", check)
    return out.value if st == VLAC_OK else st


def vlac_destroy(ctx, check=True):
    return _ret(lib().vlac_destroy(ctx), "vlac_destroy", check)


def vlac_last_hip_error(ctx):
    return lib().vlac_last_hip_error(ctx)


def vlac_set_layer_weights(ctx, layer, w, stream=None, check=True):
    """w: dict/object with bf16 GPU tensors wqkv, wo, w_gate_up, w_down, g_attn, g_ffn."""
    import torch
    get = (lambda k: w[k]) if isinstance(w, dict) else (lambda k: getattr(w, k))
    lw = LayerW(*[_ptr(get(k), torch.bfloat16, k) for k in
                  ("wqkv", "wo", "w_gate_up", "w_down", "g_attn", "g_ffn")])
    return _ret(lib().vlac_set_layer_weights(ctx, layer, C.byref(lw), _stream(stream)),
                "vlac_set_layer_weights", check)


def vlac_set_head_weights(ctx, g_final, w_head, embed, stream=None, check=True):
    import torch
    bf = torch.bfloat16
    return _ret(lib().vlac_set_head_weights(ctx, _ptr(g_final, bf, "g_final"), _ptr(w_head, bf, "w_head"),
                                            _ptr(embed, bf, "embed"), _stream(stream)),
                "vlac_set_head_weights", check)


def vlac_reset_stream(ctx, b, kv_cache, stream=None, check=True):
    return _ret(lib().vlac_reset_stream(ctx, b, _ptr(kv_cache, None, "kv_cache"), _stream(stream)),
                "vlac_reset_stream", check)


def vlac_check(ctx, stream=None, check=True):
    return _ret(lib().vlac_check(ctx, _stream(stream)), "vlac_check", check)


def vlac_profile_select(ctx, kind, check=True):
    return _ret(lib().vlac_profile_select(ctx, kind), "vlac_profile_select", check)


def vlac_profile_read(ctx, check=True):
    """Returns (total_ms, launches)."""
    ms, n = C.c_double(), C.c_int()
    _ret(lib().vlac_profile_read(ctx, C.byref(ms), C.byref(n)), "vlac_profile_read", check)
    return ms.value, n.value


def vlac_profile_bracket_cost(ctx, stream=None, check=True):
    """Microseconds that an event bracket adds to the kernel inside it."""
    us = C.c_double()
    _ret(lib().vlac_profile_bracket_cost(ctx, _stream(stream), C.byref(us)), "vlac_profile_bracket_cost", check)
    return us.value


def vlac_profile_read2(ctx, check=True):
    """Returns (total_ms, marker_ms, launches)."""
    ms, mk, n = C.c_double(), C.c_double(), C.c_int()
    _ret(lib().vlac_profile_read2(ctx, C.byref(ms), C.byref(mk), C.byref(n)), "vlac_profile_read2", check)
    return ms.value, mk.value, n.value


def vlac_select_static(ctx, frame_prev, frame_cur, B, H, W, patch, tau_num, tau_den, top_k,
                       attn_mean, layer_mask, tau_task, out_idx, out_order, out_count,
                       out_relevance, stride, stream=None, check=True):
    import torch
    mask = None
    if layer_mask is not None:
        mask = (C.c_uint8 * len(layer_mask))(*[1 if m else 0 for m in layer_mask])
    st = lib().vlac_select_static(
        ctx, _ptr(frame_prev, torch.uint8, "frame_prev"), _ptr(frame_cur, torch.uint8, "frame_cur"),
        B, H, W, patch, tau_num, tau_den, top_k, _ptr(attn_mean, torch.float32, "attn_mean"),
        C.cast(mask, C.c_void_p) if mask is not None else None, float(tau_task),
        _ptr(out_idx, torch.int32, "out_idx"), _ptr(out_order, torch.int32, "out_order"),
        _ptr(out_count, torch.int32, "out_count"), _ptr(out_relevance, torch.float32, "out_relevance"),
        stride, _stream(stream))
    return _ret(st, "vlac_select_static", check)


def vlac_select_static_noalloc(frame_prev, frame_cur, B, H, W, patch, tau_num, tau_den, top_k,
                               attn_mean, n_layers, layer_mask, tau_task, out_idx, out_order, out_count,
                               out_relevance, stride, stream=None, check=True):
    import torch
    mask = None
    if layer_mask is not None:
        mask = (C.c_uint8 * len(layer_mask))(*[1 if m else 0 for m in layer_mask])
    st = lib().vlac_select_static_noalloc(
        _ptr(frame_prev, torch.uint8, "frame_prev"), _ptr(frame_cur, torch.uint8, "frame_cur"),
        B, H, W, patch, tau_num, tau_den, top_k, _ptr(attn_mean, torch.float32, "attn_mean"), n_layers,
        C.cast(mask, C.c_void_p) if mask is not None else None, float(tau_task),
        _ptr(out_idx, torch.int32, "out_idx"), _ptr(out_order, torch.int32, "out_order"),
        _ptr(out_count, torch.int32, "out_count"), _ptr(out_relevance, torch.float32, "out_relevance"),
        stride, _stream(stream))
    return _ret(st, "vlac_select_static_noalloc", check)


def vlac_quantize_e4m3(w, out_codes, out_scales, stream=None, check=True):
    """w: bf16 GPU tensor [N, K]; out_codes uint8 [N, K]; out_scales fp32 [N]."""
    import torch
    N, K = w.shape
    st = lib().vlac_quantize_e4m3(_ptr(w, torch.bfloat16, "w"), N, K, _ptr(out_codes, torch.uint8, "out_codes"),
                                  _ptr(out_scales, torch.float32, "out_scales"), _stream(stream))
    return _ret(st, "vlac_quantize_e4m3", check)


def vlac_embed_patches(ctx, frame_cur, B, H, W, patch, w_proj, reuse_order, reuse_count, stride,
                       layer_count, embeds, L, stream=None, check=True):
    import torch
    i32 = torch.int32
    st = lib().vlac_embed_patches(
        ctx, _ptr(frame_cur, torch.uint8, "frame_cur"), B, H, W, patch,
        _ptr(w_proj, torch.bfloat16, "w_proj"), _ptr(reuse_order, i32, "reuse_order"),
        _ptr(reuse_count, i32, "reuse_count"), stride, _ptr(layer_count, i32, "layer_count"),
        _ptr(embeds, torch.float32, "embeds"), L, _stream(stream))
    return _ret(st, "vlac_embed_patches", check)


def vlac_layer_ratio(ctx, attn_mean, B, L_v, gain_k, reuse_count, out_alpha, out_layer_count,
                     stream=None, check=True):
    import torch
    st = lib().vlac_layer_ratio(
        ctx, _ptr(attn_mean, torch.float32, "attn_mean"), B, L_v, float(gain_k),
        _ptr(reuse_count, torch.int32, "reuse_count"), _ptr(out_alpha, torch.float32, "out_alpha"),
        _ptr(out_layer_count, torch.int32, "out_layer_count"), _stream(stream))
    return _ret(st, "vlac_layer_ratio", check)


def vlac_sparse_prefill(ctx, embeds, B, L_v, L_t, reuse_order, reuse_count, stride, layer_count,
                        kv_cache, out_attn_mean, out_hidden, out_logits, out_token, stream=None,
                        check=True):
    import torch
    f32, i32 = torch.float32, torch.int32
    st = lib().vlac_sparse_prefill(
        ctx, _ptr(embeds, f32, "embeds"), B, L_v, L_t, _ptr(reuse_order, i32, "reuse_order"),
        _ptr(reuse_count, i32, "reuse_count"), stride, _ptr(layer_count, i32, "layer_count"),
        _ptr(kv_cache, None, "kv_cache"), _ptr(out_attn_mean, f32, "out_attn_mean"),
        _ptr(out_hidden, f32, "out_hidden"), _ptr(out_logits, f32, "out_logits"),
        _ptr(out_token, i32, "out_token"), _stream(stream))
    return _ret(st, "vlac_sparse_prefill", check)


def vlac_decode_action(ctx, B, L, n_new, first_token, kv_cache, out_tokens, out_logits,
                       stream=None, check=True):
    import torch
    st = lib().vlac_decode_action(
        ctx, B, L, n_new, _ptr(first_token, torch.int32, "first_token"),
        _ptr(kv_cache, None, "kv_cache"), _ptr(out_tokens, torch.int32, "out_tokens"),
        _ptr(out_logits, torch.float32, "out_logits"), _stream(stream))
    return _ret(st, "vlac_decode_action", check)
