"""Host-only checks of the C ABI: the library loads, exports every function the
header declares, and rejects bad arguments before touching the GPU."""
import ctypes as C
import os
import re

import pytest

import paper_2502_02175_amd as V

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vlac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vlac_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"vlac_select_static", "vlac_layer_ratio", "vlac_sparse_prefill",
            "vlac_decode_action"} <= set(names)
    lib = V.lib()
    for n in names:
        assert hasattr(lib, n), n
    # and the Python binding carries the same names
    for n in names:
        assert hasattr(V, n) or n == "vlac_status_string", n


def test_status_strings():
    assert V.status_string(0) == "ok"
    for s in range(-6, 0):
        assert V.status_string(s) not in ("ok", "unknown status")
    assert V.status_string(-99) == "unknown status"


def good_cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=688,
                vocab=256, rms_eps=1e-6, rope_base=1e4, max_batch=2, max_seq=96, operand_dtype=0)
    base.update(kw)
    return V.ModelCfg(**base)


def test_create_rejects_bad_shapes_on_the_host():
    out = C.c_void_p()
    lib = V.lib()
    assert lib.vlac_create(None, C.byref(out)) == -1
    assert lib.vlac_create(C.byref(good_cfg()), None) == -1
    for kw, want in ((dict(head_dim=96), -2), (dict(d_model=250), -2), (dict(d_ffn=100), -2),
                     (dict(vocab=100), -2), (dict(max_seq=100), -2), (dict(n_q_heads=6), -2),
                     (dict(n_q_heads=8, n_kv_heads=3), -2), (dict(n_layers=0), -3),
                     (dict(max_batch=0), -3), (dict(max_seq=1 << 20), -3), (dict(rms_eps=0.0), -3),
                     (dict(rope_base=1.0), -3), (dict(operand_dtype=3), -3)):
        cfg = good_cfg(**kw)
        assert lib.vlac_create(C.byref(cfg), C.byref(out)) == want, kw
        assert V.vlac_kv_cache_bytes(cfg) == 0
    assert out.value is None


def test_kv_cache_bytes():
    cfg = good_cfg()
    assert V.vlac_kv_cache_bytes(cfg) == 2 * 2 * 2 * 4 * 96 * 64 * 2   # streams*layers*(K,V)*heads*seq*hd*2B


def test_null_context_is_rejected():
    lib = V.lib()
    assert lib.vlac_destroy(None) == -1
    assert lib.vlac_check(None, None) == -1
    assert lib.vlac_layer_ratio(None, None, 1, 1, 1.0, None, None, None, None) == -1
    assert lib.vlac_decode_action(None, 1, 1, 1, None, None, None, None, None) == -1
    assert lib.vlac_sparse_prefill(None, None, 1, 1, 1, None, None, 1, None, None, None, None, None,
                                   None, None) == -1


def test_entry_points_beside_the_path_reject_null_arguments():
    lib = V.lib()
    assert lib.vlac_embed_patches(None, None, 1, 14, 14, 14, None, None, None, 1, None, None, 1, None) == -1
    assert lib.vlac_quantize_e4m3(None, 4, 8, None, None, None) == -1
    assert lib.vlac_profile_read2(None, None, None, None) == -1
    assert lib.vlac_profile_bracket_cost(None, None, None) == -1
    assert lib.vlac_select_static(None, None, None, 1, 14, 14, 14, 249, 250, 1, None, None, 0.5,
                                  None, None, None, None, 1, None) == -1


def test_no_cpu_fallback_without_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    st = V.vlac_create(good_cfg(), check=False)
    assert st < 0          # fails loudly: there is no CPU path
