"""GPU parity at the benchmark's shape (OpenVLA-7B decoder dims, 256 visual + 32
text tokens, 77 of 256 patches re-drawn, top-k 180), in the launch configuration
bench.py times (one stream, worst-case grids, device-side row counts).

The oracle finishes a few layers of this shape in seconds, so element-wise
parity runs on the first 3 layers; at the full depth of 32 layers the test
checks properties that hold at any size."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from helpers import GpuModel, oracle_model

pytestmark = pytest.mark.gpu
# fp16 operands: the stated bar, max-abs 2e-2.  bf16 operands cannot meet it at this
# shape: a pipeline that does nothing but round the same tensors to bf16 (every
# sum exact) is already 3.7e-2 away from the fp64 result after 3 layers, because
# each rounding (2^-9 relative) is amplified by the random-init layers that follow.
# Its bar here is twice that figure.
TOLS = {"f16": 2e-2, "bf16": 8e-2}
CFG = synth.CONFIGS["7b"]
H, PATCH, N_VIS, N_TXT, TOP_K, N_REDRAW = 224, 14, 256, 32, 180, 77
L = N_VIS + N_TXT


def inputs(seed):
    prev, cur, redrawn = synth.frame_pair(H, H, PATCH, N_REDRAW, seed)
    wp = synth.projection_matrix(CFG.d_model, PATCH, seed + 1)
    txt = synth.round_bf16(synth.text_embeddings(N_TXT, CFG.d_model, seed + 2))
    e_prev = np.concatenate([synth.round_bf16(synth.visual_embeddings(prev, PATCH, wp)), txt])
    e_cur = np.concatenate([synth.round_bf16(synth.visual_embeddings(cur, PATCH, wp)), txt])
    return prev, cur, redrawn, e_prev, e_cur


def margin(x):
    s = np.sort(np.asarray(x, dtype=np.float64))
    return s[-1] - s[-2]


@pytest.mark.parametrize("operand", ["f16", "bf16"])
def test_7b_shape_three_layers_against_oracle(operand):
    TOL = TOLS[operand]
    cfg = CFG.with_layers(3)
    prev, cur, redrawn, e_prev, e_cur = inputs(seed=0)
    om = oracle_model(cfg, seed=0, gain_jitter=0.1)
    gm = GpuModel(cfg, seed=0, max_batch=1, max_seq=320, gain_jitter=0.1, operand=operand)
    try:
        cache = O.new_cache(cfg, 320)
        want1 = O.dense_forward(om, e_prev, N_VIS, cache)
        got1 = gm.prefill(e_prev[None], N_VIS)
        e_h = np.abs(got1["hidden"][0] - want1["hidden"]).max()
        e_l = np.abs(got1["logits"][0] - want1["logits"]).max()
        print("\n[%s] full prefill: max-abs hidden %.4g logits %.4g" % (operand, e_h, e_l))
        assert e_h <= TOL and e_l <= TOL
        np.testing.assert_allclose(got1["attn_mean"][:, 0], want1["attn_mean"], atol=1e-4, rtol=2e-2)

        # Alg. 1 on the GPU against the oracle (bit-exact), filter on the oracle's statistics
        sel = gm.select(prev[None], cur[None], PATCH, 249, 250, TOP_K, want1["attn_mean"][:, None], 1.0)
        p_static = O.select_static(prev, cur, PATCH, 249, 250, TOP_K)
        assert sel["idx"][0] == p_static == [i for i in range(N_VIS) if not redrawn[i]]
        assert len(p_static) == 179

        want2 = O.sparse_forward(om, e_cur, N_VIS, cache, [p_static] * cfg.n_layers)
        got2 = gm.prefill(e_cur[None], N_VIS, [sel["order"][0]])
        alive = ~np.isnan(want2["hidden"][:, 0])
        assert alive.sum() == L - 179
        e_h = np.abs(got2["hidden"][0][alive] - want2["hidden"][alive]).max()
        e_l = np.abs(got2["logits"][0] - want2["logits"]).max()
        print("[%s] sparse prefill: max-abs hidden %.4g logits %.4g" % (operand, e_h, e_l))
        assert e_h <= TOL and e_l <= TOL
        assert np.all(np.isnan(got2["hidden"][0][~alive]))
        np.testing.assert_allclose(got2["attn_mean"][:, 0], want2["attn_mean"], atol=1e-4, rtol=2e-2)
        if margin(want2["logits"]) > 2 * TOL:
            assert int(got2["token"][0]) == want2["token"]

        toks, logits = O.decode(om, cache, L, want2["token"], 2, return_logits=True)
        gt, gl = gm.decode(1, L, 2, [want2["token"]])
        assert np.abs(gl[0] - logits).max() <= TOL
        if all(margin(x) > 2 * TOL for x in logits):
            assert gt[0].tolist() == toks
    finally:
        gm.close()


def test_7b_full_depth_properties():
    """32 layers (weights drawn on the GPU; nothing here is compared with the CPU):
    identical frames => sparse prefill equals the full recompute (cached K/V are
    exactly what recomputation gives; rows are independent in every kernel, so the
    equality is bit for bit); an empty reuse list equals the full recompute;
    reused cache rows are untouched; 6 decoded tokens are reproducible."""
    import torch
    prev, cur, redrawn, e_prev, e_cur = inputs(seed=1)
    gm = GpuModel(CFG, seed=1, max_batch=1, max_seq=320, gain_jitter=0.1, gen_device="cuda:0")
    try:
        static = [i for i in range(N_VIS) if not redrawn[i]]
        full = gm.prefill(e_cur[None], N_VIS)
        t_full, _ = gm.decode(1, L, 6, full["token"])
        assert np.isfinite(full["logits"]).all() and np.isfinite(full["hidden"]).all()
        same = gm.prefill(e_cur[None], N_VIS, [static])          # same frame again, 179 reused
        np.testing.assert_array_equal(same["logits"], full["logits"])
        # (the statistic sums the same text rows in another lane order: equal up to fp32 rounding)
        np.testing.assert_allclose(same["attn_mean"], full["attn_mean"], rtol=1e-4, atol=1e-8)
        alive = np.array([i not in set(static) for i in range(L)])
        np.testing.assert_array_equal(same["hidden"][0][alive], full["hidden"][0][alive])
        t_same, _ = gm.decode(1, L, 6, same["token"])
        np.testing.assert_array_equal(t_same, t_full)
        empty = gm.prefill(e_cur[None], N_VIS, [[]])
        np.testing.assert_array_equal(empty["logits"], full["logits"])
        # a changed frame with reuse: reused rows of the cache keep their bytes, and the
        # result differs from the full recompute of the new frame (how far says nothing
        # with random-init weights, which amplify any perturbation over 32 layers)
        gm.prefill(e_prev[None], N_VIS)
        kv_before = gm.kv.clone()
        sparse = gm.prefill(e_cur[None], N_VIS, [static])
        changed = (gm.kv != kv_before).sum().item()
        # recomputed rows: (L - 179) positions x 32 layers x (K and V) x 4096 features x 2 bytes
        assert 0 < changed <= (L - 179) * 32 * 2 * 4096 * 2
        full2 = gm.prefill(e_cur[None], N_VIS)
        d = np.abs(sparse["logits"] - full2["logits"]).max()
        assert d > 0 and np.isfinite(sparse["logits"]).all()
        del kv_before
        torch.cuda.empty_cache()
    finally:
        gm.close()
