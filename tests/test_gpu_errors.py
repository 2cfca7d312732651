"""The argument checks of the C ABI that need a context (and so a GPU): every documented
host-side error is returned with its status, and a refused call queues nothing (its output
buffers still hold what the caller put there after the stream has drained).  Alg. 1 inputs
and hyper-parameters: Sec. 3.2 / 3.3; Alg. 2: the reuse lists and the cache state."""
import ctypes as C

import numpy as np
import pytest

import synth
import paper_2502_02175_amd as V

pytestmark = pytest.mark.gpu
E_NULL, E_SHAPE, E_RANGE, E_STATE = -1, -2, -3, -4
CFG = synth.CONFIGS["tiny"]


@pytest.fixture(scope="module")
def env():
    import torch
    dev = "cuda:0"
    ccfg = V.ModelCfg(CFG.n_layers, CFG.d_model, CFG.n_q_heads, CFG.n_kv_heads, CFG.head_dim, CFG.d_ffn,
                      CFG.vocab, CFG.rms_eps, CFG.rope_base, 2, 96, 1)
    ctx = V.vlac_create(ccfg)
    kv = torch.zeros(V.vlac_kv_cache_bytes(ccfg), dtype=torch.uint8, device=dev)
    t = dict(
        torch=torch, ctx=ctx, kv=kv, ccfg=ccfg,
        frames=torch.zeros((2, 2, 112, 112, 3), dtype=torch.uint8, device=dev),
        idx=torch.full((2, 64), -7, dtype=torch.int32, device=dev),
        order=torch.full((2, 64), -7, dtype=torch.int32, device=dev),
        count=torch.full((2,), -7, dtype=torch.int32, device=dev),
        stats=torch.full((CFG.n_layers, 2, 64), 1.0 / 64, device=dev),
        alpha=torch.full((2, CFG.n_layers), -7.0, device=dev),
        lcount=torch.full((2, CFG.n_layers), -7, dtype=torch.int32, device=dev),
        emb=torch.zeros((2, 80, CFG.d_model), device=dev),
        logits=torch.full((2, CFG.vocab), -7.0, device=dev),
        token=torch.full((2,), -7, dtype=torch.int32, device=dev),
        toks=torch.full((2, 4), -7, dtype=torch.int32, device=dev),
    )
    yield t
    V.vlac_destroy(ctx)


def untouched(t):
    t["torch"].cuda.synchronize()
    for k in ("idx", "order", "count", "lcount", "token", "toks"):
        assert bool((t[k] == -7).all()), k
    assert bool((t["alpha"] == -7.0).all()) and bool((t["logits"] == -7.0).all())


def select(t, B=1, H=112, W=112, patch=14, num=249, den=250, k=32, stats=None, tau_task=0.5, stride=64):
    return V.vlac_select_static(t["ctx"], t["frames"][0], t["frames"][1], B, H, W, patch, num, den, k,
                                stats, None, tau_task, t["idx"], t["order"], t["count"], None, stride,
                                check=False)


def test_select_static_argument_checks(env):
    t = env
    assert select(t, H=110) == E_SHAPE and select(t, W=100) == E_SHAPE          # H, W multiples of patch
    assert select(t, den=0) == E_RANGE and select(t, den=-5) == E_RANGE
    assert select(t, num=-1) == E_RANGE and select(t, num=251) == E_RANGE     # 0 <= tau <= 1
    assert select(t, k=-1) == E_RANGE and select(t, k=65) == E_RANGE          # 0 <= top_k <= L_v
    assert select(t, k=32, stride=31) == E_SHAPE and select(t, k=0, stride=0) == E_SHAPE
    assert select(t, B=0) == E_RANGE and select(t, B=3) == E_RANGE            # max_batch is 2
    assert select(t, patch=0) == E_RANGE and select(t, patch=65, H=130, W=130) == E_RANGE
    assert select(t, patch=1, H=112, W=112) == E_RANGE                        # 12544 patches > 4096
    assert select(t, stats=t["stats"], tau_task=float("nan")) == E_RANGE
    assert V.vlac_select_static(t["ctx"], t["frames"][0], None, 1, 112, 112, 14, 249, 250, 32, None, None,
                                0.5, t["idx"], t["order"], t["count"], None, 64, check=False) == E_NULL
    assert V.vlac_select_static(t["ctx"], t["frames"][0], t["frames"][1], 1, 112, 112, 14, 249, 250, 32, None,
                                None, 0.5, t["idx"], None, t["count"], None, 64, check=False) == E_NULL
    untouched(t)


def test_layer_ratio_argument_checks(env):
    t = env
    lr = lambda B=1, L_v=64, gain=1.0, rc=t["count"], alpha=t["alpha"], lc=t["lcount"], stats=t["stats"]: \
        V.vlac_layer_ratio(t["ctx"], stats, B, L_v, gain, rc, alpha, lc, check=False)
    assert lr(B=0) == E_RANGE and lr(B=3) == E_RANGE
    assert lr(L_v=0) == E_RANGE and lr(L_v=70000) == E_RANGE
    assert lr(gain=float("nan")) == E_RANGE
    assert lr(rc=None) == E_NULL                       # per-layer counts need the reuse count
    assert lr(alpha=None) == E_NULL and lr(stats=None) == E_NULL
    untouched(t)


def prefill(t, B=1, L_v=64, L_t=16, order="x", count="x", stride=64, lc=None, kv="x", token="x", emb="x"):
    g = lambda v, k: t[k] if isinstance(v, str) else v
    return V.vlac_sparse_prefill(t["ctx"], g(emb, "emb"), B, L_v, L_t, g(order, "order"), g(count, "count"),
                                 stride, lc, g(kv, "kv"), None, None, t["logits"], g(token, "token"),
                                 check=False)


def decode(t, B=1, L=80, n_new=2, first="x", kv="x", out="x"):
    g = lambda v, k: t[k] if isinstance(v, str) else v
    return V.vlac_decode_action(t["ctx"], B, L, n_new, g(first, "count"), g(kv, "kv"), g(out, "toks"), None,
                                check=False)


def test_prefill_and_decode_argument_and_state_checks(env):
    t = env
    torch, ctx = t["torch"], t["ctx"]
    # shape and range checks come before the state checks
    assert prefill(t, B=0) == E_RANGE and prefill(t, B=3) == E_RANGE
    assert prefill(t, L_v=-1) == E_RANGE and prefill(t, L_v=0, L_t=0) == E_RANGE
    assert prefill(t, L_v=64, L_t=40) == E_SHAPE                    # 104 tokens > max_seq 96
    assert prefill(t, stride=0) == E_SHAPE and prefill(t, L_v=0, L_t=16) == E_SHAPE   # lists need visual tokens
    assert prefill(t, order=None) == E_NULL and prefill(t, count=None) == E_NULL      # both or neither
    assert prefill(t, order=None, count=None, lc=t["lcount"]) == E_NULL
    assert prefill(t, kv=None) == E_NULL and prefill(t, token=None) == E_NULL and prefill(t, emb=None) == E_NULL
    assert decode(t, B=0) == E_RANGE and decode(t, B=3) == E_RANGE and decode(t, L=0) == E_RANGE
    assert decode(t, n_new=-1) == E_RANGE
    assert decode(t, L=90, n_new=7) == E_SHAPE                      # L + n_new > max_seq
    assert decode(t, first=None) == E_NULL and decode(t, kv=None) == E_NULL and decode(t, out=None) == E_NULL
    # state: weights missing
    assert prefill(t, order=None, count=None) == E_STATE and decode(t) == E_STATE
    for l in range(CFG.n_layers):
        w = {k: v.to("cuda:0") for k, v in synth.make_layer(CFG, 0, l).items()}
        V.vlac_set_layer_weights(ctx, l, w)
        torch.cuda.synchronize()
    assert prefill(t, order=None, count=None) == E_STATE            # the head is still missing
    hd = {k: v.to("cuda:0") for k, v in synth.make_head(CFG, 0).items()}
    assert V.vlac_set_layer_weights(ctx, CFG.n_layers, w, check=False) == E_RANGE
    assert V.lib().vlac_set_layer_weights(ctx, 0, None, None) == E_NULL
    lw = V.LayerW(*[w[k].data_ptr() for k in ("wqkv", "wo", "w_gate_up", "w_down", "g_attn")], None)
    assert V.lib().vlac_set_layer_weights(ctx, 0, C.byref(lw), None) == E_NULL
    assert V.vlac_set_head_weights(ctx, hd["g_final"], None, hd["embed"], check=False) == E_NULL
    V.vlac_set_head_weights(ctx, hd["g_final"], hd["w_head"], hd["embed"])
    torch.cuda.synchronize()
    # state: a stream that was never reset; then one whose cache holds no prefill yet
    assert prefill(t, order=None, count=None) == E_STATE
    assert V.vlac_reset_stream(ctx, 2, t["kv"], check=False) == E_RANGE
    assert V.vlac_reset_stream(ctx, -1, t["kv"], check=False) == E_RANGE
    assert V.vlac_reset_stream(ctx, 0, None, check=False) == E_NULL
    V.vlac_reset_stream(ctx, 0, t["kv"])
    assert prefill(t) == E_STATE                                    # reuse lists before any full prefill
    assert decode(t) == E_STATE
    assert prefill(t, B=2, order=None, count=None) == E_STATE       # stream 1 was not reset
    untouched(t)
    # and the same calls go through once the state is there
    assert prefill(t, order=None, count=None) == 0
    t["count"].fill_(0)
    assert prefill(t) == 0 and decode(t) == 0
    assert V.vlac_check(ctx) == 0
    assert decode(t, B=2) == E_STATE                                # stream 1 still holds nothing
    torch.cuda.synchronize()
    assert int(t["token"][0]) >= 0 and int(t["token"][1]) == -7
    # after a reset the stream needs a full prefill again
    V.vlac_reset_stream(ctx, 0, t["kv"])
    assert prefill(t) == E_STATE and decode(t) == E_STATE


def test_embed_patches_argument_checks(env):
    t = env
    torch = t["torch"]
    wp = torch.zeros((588, CFG.d_model), dtype=torch.bfloat16, device="cuda:0")
    ep = lambda B=1, H=112, W=112, patch=14, w=wp, order=None, count=None, stride=64, L=80: \
        V.vlac_embed_patches(t["ctx"], t["frames"][1], B, H, W, patch, w, order, count, stride, None,
                             t["emb"], L, check=False)
    assert ep(B=3) == E_RANGE and ep(B=0) == E_RANGE
    assert ep(patch=27, H=108, W=108) == E_SHAPE and ep(H=110) == E_SHAPE
    assert ep(L=63) == E_SHAPE                                       # fewer rows than patches
    assert ep(w=None) == E_NULL
    assert ep(order=t["order"]) == E_NULL                            # list without its count
    assert ep(order=t["order"], count=t["count"], stride=0) == E_RANGE
