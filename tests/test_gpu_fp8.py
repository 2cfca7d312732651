"""Weight-only e4m3 storage (operand mode F16_W8) on the GPU: the quantiser bit for bit
against the oracle's, and the whole path (prefill, sparse prefill, decode) against the
oracle run on the weights as the oracle's quantiser keeps them.  Tolerance as everywhere:
max-abs 2e-2 on hidden states and logits (the arithmetic is that of the F16 mode, the
expansion of the codes to fp16 is exact)."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from oracle import fp8 as Q
from helpers import GpuModel, oracle_model, tiny_inputs

pytestmark = pytest.mark.gpu
TOL = 2e-2
TINY = synth.CONFIGS["tiny"]


def margin(logits):
    s = np.sort(np.asarray(logits, dtype=np.float64))
    return s[-1] - s[-2]


def test_quantiser_matches_oracle_bit_for_bit():
    import torch
    import paper_2502_02175_amd as V
    rng = np.random.default_rng(0)
    N, K = 96, 520
    w = rng.standard_normal((N, K)) * 0.02
    w[0] = 0.0                                   # zero row: scale 1, codes 0
    w[1, :] = 448.0 * 2.0 ** -9                  # the row maximum exactly at the top of a scale
    w[2, 0] = 448.0 * 2.0 ** -9 * 1.004          # just above it: the next scale (bf16 keeps the excess)
    w[3] *= 1e-6
    w[4, :127] = Q._POS * 2.0 ** -3              # every representable value ...
    w[5, :126] = (Q._POS[:-1] + Q._POS[1:]) / 2 * 2.0 ** -3   # ... and every tie
    w[5, 126] = 448.0 * 2.0 ** -3
    w[6] = -w[5]
    w = synth.round_bf16(w).astype(np.float32)   # what the library is handed
    d_w = torch.tensor(w, device="cuda").to(torch.bfloat16)
    codes = torch.zeros((N, K), dtype=torch.uint8, device="cuda")
    scales = torch.zeros(N, device="cuda")
    V.vlac_quantize_e4m3(d_w, codes, scales)
    torch.cuda.synchronize()
    want_codes, want_scales, _ = Q.quantize_rows(w)
    np.testing.assert_array_equal(scales.cpu().numpy().astype(np.float64), want_scales)
    got = codes.cpu().numpy()
    # (+0 and -0 are the same weight)
    same = (got == want_codes) | (((got & 0x7F) == 0) & ((want_codes & 0x7F) == 0))
    assert same.all(), np.argwhere(~same)[:5]


def test_tiny_path_with_e4m3_weights():
    prev, cur, redrawn, e_prev, e_cur = tiny_inputs(seed=0)
    om = oracle_model(TINY, seed=0, std=0.05, w8=True)
    plain = oracle_model(TINY, seed=0, std=0.05)
    gm = GpuModel(TINY, seed=0, max_batch=2, max_seq=96, std=0.05, operand="f16w8")
    try:
        cache = O.new_cache(TINY, 96)
        want1 = O.dense_forward(om, e_prev, 64, cache)
        got1 = gm.prefill(e_prev[None], 64)
        assert np.abs(got1["hidden"][0] - want1["hidden"]).max() <= TOL
        assert np.abs(got1["logits"][0] - want1["logits"]).max() <= TOL
        # the quantised model is a different model: the unquantised oracle is far outside the tolerance
        far = O.dense_forward(plain, e_prev, 64, O.new_cache(TINY, 96))
        assert np.abs(got1["logits"][0] - far["logits"]).max() > 2 * TOL
        p_final, order, per_layer, alpha = O.plan_step(prev, cur, 14, 249, 250, 32, want1["attn_mean"], 0.5, 2.0)
        want2 = O.sparse_forward(om, e_cur, 64, cache, per_layer)
        got2 = gm.prefill(e_cur[None], 64, [order], [[len(s) for s in per_layer]])
        alive = ~np.isnan(want2["hidden"][:, 0])
        assert np.abs(got2["hidden"][0][alive] - want2["hidden"][alive]).max() <= TOL
        assert np.abs(got2["logits"][0] - want2["logits"]).max() <= TOL
        np.testing.assert_allclose(got2["attn_mean"][:, 0], want2["attn_mean"], atol=2e-4, rtol=2e-2)
        toks, logits = O.decode(om, cache, 80, want2["token"], 3, return_logits=True)
        gt, gl = gm.decode(1, 80, 3, [want2["token"]])
        assert np.abs(gl[0] - logits).max() <= TOL
        if all(margin(l) > 2 * TOL for l in logits) and margin(want2["logits"]) > 2 * TOL:
            assert int(got2["token"][0]) == want2["token"] and gt[0].tolist() == toks
        # two streams at once (the few-rows kernels without the fused norm are not used at B <= 4;
        # B = 2 still runs them for the prefill's head)
        got_b = gm.prefill(np.stack([e_prev, e_cur]), 64)
        assert np.abs(got_b["logits"][0] - want1["logits"]).max() <= TOL
    finally:
        gm.close()


def test_7b_shape_three_layers_with_e4m3_weights():
    cfg = synth.CONFIGS["7b"].with_layers(3)
    H, PATCH, N_VIS, N_TXT, TOP_K, N_REDRAW = 224, 14, 256, 32, 180, 77
    L = N_VIS + N_TXT
    prev, cur, redrawn = synth.frame_pair(H, H, PATCH, N_REDRAW, 1)
    wp = synth.projection_matrix(cfg.d_model, PATCH, 2)
    txt = synth.round_bf16(synth.text_embeddings(N_TXT, cfg.d_model, 3))
    e_prev = np.concatenate([synth.round_bf16(synth.visual_embeddings(prev, PATCH, wp)), txt])
    e_cur = np.concatenate([synth.round_bf16(synth.visual_embeddings(cur, PATCH, wp)), txt])
    om = oracle_model(cfg, seed=1, gain_jitter=0.1, w8=True)
    gm = GpuModel(cfg, seed=1, max_batch=1, max_seq=320, gain_jitter=0.1, operand="f16w8")
    try:
        cache = O.new_cache(cfg, 320)
        want = O.dense_forward(om, e_prev, N_VIS, cache)
        got = gm.prefill(e_prev[None], N_VIS)
        e_h = np.abs(got["hidden"][0] - want["hidden"]).max()
        e_l = np.abs(got["logits"][0] - want["logits"]).max()
        print("\nfull prefill: max-abs hidden %.4g logits %.4g" % (e_h, e_l))
        assert e_h <= TOL and e_l <= TOL
        p_static = O.select_static(prev, cur, PATCH, 249, 250, TOP_K)
        want2 = O.sparse_forward(om, e_cur, N_VIS, cache, [p_static] * cfg.n_layers)
        got2 = gm.prefill(e_cur[None], N_VIS, [p_static])
        alive = ~np.isnan(want2["hidden"][:, 0])
        e_h = np.abs(got2["hidden"][0][alive] - want2["hidden"][alive]).max()
        e_l = np.abs(got2["logits"][0] - want2["logits"]).max()
        print("sparse prefill: max-abs hidden %.4g logits %.4g" % (e_h, e_l))
        assert e_h <= TOL and e_l <= TOL
        toks, logits = O.decode(om, cache, L, want2["token"], 2, return_logits=True)
        gt, gl = gm.decode(1, L, 2, [want2["token"]])
        assert np.abs(gl[0] - logits).max() <= TOL
        if all(margin(x) > 2 * TOL for x in logits):
            assert gt[0].tolist() == toks
    finally:
        gm.close()


@pytest.mark.parametrize("B", [8, 16])
def test_many_rows_with_e4m3_weights(B):
    """16 streams at once: 1280 rows go to the many-rows GEMM, which has no variant for the
    codes and gets every matrix expanded to fp16 before its launch (8 streams: 640 rows stay
    with the one-stream kernel, five row blocks of it); a full and a sparse prefill against
    the oracle on the quantised weights."""
    prev, cur, redrawn, e_prev, e_cur = tiny_inputs(seed=0)
    om = oracle_model(TINY, seed=0, std=0.05, w8=True)
    gm = GpuModel(TINY, seed=0, max_batch=B, max_seq=96, std=0.05, operand="f16w8")
    try:
        cache_p, cache_c = O.new_cache(TINY, 96), O.new_cache(TINY, 96)
        want_p = O.dense_forward(om, e_prev, 64, cache_p)
        want_c = O.dense_forward(om, e_cur, 64, cache_c)
        got = gm.prefill(np.stack([e_prev, e_cur] * (B // 2)), 64)
        for b in range(B):
            want = want_p if b % 2 == 0 else want_c
            assert np.abs(got["hidden"][b] - want["hidden"]).max() <= TOL, b
            assert np.abs(got["logits"][b] - want["logits"]).max() <= TOL, b
        # every stream moves on to the current frame: the even ones reuse the static tokens of
        # the frame pair, the odd ones (same frame again) every second token
        p_static = O.select_static(prev, cur, 14, 249, 250, 32)
        want_s = O.sparse_forward(om, e_cur, 64, cache_p, [p_static] * TINY.n_layers)
        half = list(range(0, 64, 2))
        got2 = gm.prefill(np.stack([e_cur] * B), 64, [list(p_static) if b % 2 == 0 else half for b in range(B)])
        alive = ~np.isnan(want_s["hidden"][:, 0])
        for b in range(B):
            if b % 2 == 0:
                assert np.abs(got2["hidden"][b][alive] - want_s["hidden"][alive]).max() <= TOL, b
                assert np.abs(got2["logits"][b] - want_s["logits"]).max() <= TOL, b
            else:
                assert np.abs(got2["logits"][b] - want_c["logits"]).max() <= TOL, b
    finally:
        gm.close()
