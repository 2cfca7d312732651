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
    identical frames => a sparse prefill equals the recompute of every row (cached K/V are
    exactly what recomputation gives; rows are independent in every kernel, so the
    equality is bit for bit, whatever is reused, as long as the same GEMM kernel serves: the
    reference is the prefill with an EMPTY reuse list, whose row count the kernels read from
    device memory like any sparse prefill's); the full recompute proper, whose row count the
    host knows, runs the many-rows GEMM at this size and agrees to rounding; reused cache rows
    are untouched; 6 decoded tokens are reproducible."""
    import torch
    prev, cur, redrawn, e_prev, e_cur = inputs(seed=1)
    gm = GpuModel(CFG, seed=1, max_batch=1, max_seq=320, gain_jitter=0.1, gen_device="cuda:0")
    try:
        static = [i for i in range(N_VIS) if not redrawn[i]]
        host_full = gm.prefill(e_cur[None], N_VIS)
        full = gm.prefill(e_cur[None], N_VIS, [[]])
        t_full, _ = gm.decode(1, L, 6, full["token"])
        assert np.isfinite(full["logits"]).all() and np.isfinite(full["hidden"]).all()
        # (both are within 1.5e-2 of the oracle at this depth, tests/test_gpu_depth.py)
        np.testing.assert_allclose(host_full["logits"], full["logits"], atol=3e-2)
        np.testing.assert_allclose(host_full["attn_mean"], full["attn_mean"], rtol=5e-2, atol=1e-5)
        same = gm.prefill(e_cur[None], N_VIS, [static])          # same frame again, 179 reused
        np.testing.assert_array_equal(same["logits"], full["logits"])
        # (the statistic sums the same text rows in another lane order: equal up to fp32 rounding)
        np.testing.assert_allclose(same["attn_mean"], full["attn_mean"], rtol=1e-4, atol=1e-8)
        alive = np.array([i not in set(static) for i in range(L)])
        np.testing.assert_array_equal(same["hidden"][0][alive], full["hidden"][0][alive])
        t_same, _ = gm.decode(1, L, 6, same["token"])
        np.testing.assert_array_equal(t_same, t_full)
        # ... and so does any prefix of the static set: 1 to 9 row tiles, one to three row
        # blocks (every specialisation of the GEMM main loops, their last steps included)
        for k in (256, 240, 150, 100, 40, 20):
            part = gm.prefill(e_cur[None], N_VIS, [list(range(k))], want_hidden=False)
            np.testing.assert_array_equal(part["logits"], full["logits"])
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


def test_split_k_hand_over_is_reproducible():
    """The same sparse prefills 400 times over at full depth: every one reproduces the full
    recompute bit for bit.  (Partial sums that a workgroup parks for the last one to arrive
    must have reached the memory side before the arrival counter moves; when the wait for
    that was missing, about one prefill in 400 read a stale partial tile.)"""
    prev, cur, redrawn, e_prev, e_cur = inputs(seed=2)
    gm = GpuModel(CFG, seed=2, max_batch=1, max_seq=320, gain_jitter=0.1, gen_device="cuda:0")
    try:
        # (reference: every row recomputed with the row count read on the device, as in the loop;
        # a stream's first prefill has to be a full one)
        gm.prefill(e_cur[None], N_VIS, want_stats=False, want_hidden=False)
        full = gm.prefill(e_cur[None], N_VIS, [[]], want_stats=False, want_hidden=False)["logits"]
        assert np.isfinite(full).all()
        for it in range(50):
            for k in (256, 240, 179, 150, 100, 40, 20, 0):
                part = gm.prefill(e_cur[None], N_VIS, [list(range(k))], want_stats=False, want_hidden=False)
                assert np.array_equal(part["logits"], full), (it, k)
    finally:
        gm.close()


def _random_streams(cfg, B, n_vis, n_txt, static_frac, seed):
    """Embeddings of two consecutive steps for B streams: a fraction of the visual
    tokens keeps its embedding, the rest is re-drawn."""
    rng = np.random.default_rng(seed)
    L_ = n_vis + n_txt
    e0 = synth.round_bf16(rng.standard_normal((B, L_, cfg.d_model)))
    e1 = e0.copy()
    changed = rng.random((B, n_vis)) >= static_frac
    e1[:, :n_vis][changed] = synth.round_bf16(rng.standard_normal((int(changed.sum()), cfg.d_model)))
    return e0, e1, changed


def _check_streams(cfg, B, n_vis, n_txt, static_frac, seed, n_new, tol=2e-2):
    om = oracle_model(cfg, seed=seed, gain_jitter=0.1)
    L_ = n_vis + n_txt
    max_seq = (L_ + n_new + 31) // 32 * 32
    gm = GpuModel(cfg, seed=seed, max_batch=B, max_seq=max_seq, gain_jitter=0.1)
    try:
        e0, e1, changed = _random_streams(cfg, B, n_vis, n_txt, static_frac, seed)
        caches = [O.new_cache(cfg, max_seq) for _ in range(B)]
        want0 = [O.dense_forward(om, e0[b], n_vis, caches[b]) for b in range(B)]
        got0 = gm.prefill(e0, n_vis)
        for b in range(B):
            assert np.abs(got0["hidden"][b] - want0[b]["hidden"]).max() <= tol
            assert np.abs(got0["logits"][b] - want0[b]["logits"]).max() <= tol
            np.testing.assert_allclose(got0["attn_mean"][:, b], want0[b]["attn_mean"], atol=1e-4, rtol=2e-2)
        reuse = [np.flatnonzero(~changed[b]).tolist() for b in range(B)]
        want1 = [O.sparse_forward(om, e1[b], n_vis, caches[b], [reuse[b]] * cfg.n_layers) for b in range(B)]
        got1 = gm.prefill(e1, n_vis, reuse)
        for b in range(B):
            alive = ~np.isnan(want1[b]["hidden"][:, 0])
            assert np.abs(got1["hidden"][b][alive] - want1[b]["hidden"][alive]).max() <= tol
            assert np.all(np.isnan(got1["hidden"][b][~alive]))
            assert np.abs(got1["logits"][b] - want1[b]["logits"]).max() <= tol
            np.testing.assert_allclose(got1["attn_mean"][:, b], want1[b]["attn_mean"], atol=1e-4, rtol=2e-2)
            if margin(want1[b]["logits"]) > 2 * tol:
                assert int(got1["token"][b]) == want1[b]["token"]
        first = [w["token"] for w in want1]
        gt, gl = gm.decode(B, L_, n_new, first)
        for b in range(B):
            toks, logits = O.decode(om, caches[b], L_, first[b], n_new, return_logits=True)
            assert np.abs(gl[b] - logits).max() <= tol
            if all(margin(x) > 2 * tol for x in logits):
                assert gt[b].tolist() == toks
    finally:
        gm.close()


def test_hires_batched_shape_against_oracle():
    """High-resolution batched shape: 7B layer dims, 1024 visual + 32 text tokens per
    stream, 70% static; 2 streams and 1 layer keep the oracle within seconds.  Many
    row blocks per GEMM, 33 key tiles per query, a 1024-wide attention statistic."""
    _check_streams(CFG.with_layers(1), B=2, n_vis=1024, n_txt=32, static_frac=0.7, seed=3, n_new=1)


def test_hires_batched_streams_with_few_and_many_rows():
    """The same shape with one stream 70% static (339 rows to recompute) and one 97% static
    (about 60 rows): the two attention kernels for long sequences (one query tile per wave
    for streams with 65 rows or more, one per workgroup for the others) share a launch pair."""
    _check_streams(CFG.with_layers(1), B=2, n_vis=1024, n_txt=32, static_frac=np.array([[0.7], [0.97]]),
                   seed=13, n_new=1)


@pytest.mark.parametrize("static_frac", [0.8, 0.2])
def test_two_streams_share_a_pass_with_few_or_many_rows(static_frac):
    """Two 7B-shaped streams of 288 tokens (a capacity of 576 rows, 2 layers): for a GEMM of
    such a pass both the one-stream and the many-rows kernel are launched, and the row count
    on the device says which of them works (80% static: 180 rows, the one-stream kernel and
    its 8 split-K partial rows; 20% static: 470 rows, the many-rows kernel and its plan)."""
    _check_streams(CFG.with_layers(2), B=2, n_vis=256, n_txt=32, static_frac=static_frac, seed=21, n_new=1)


def test_gqa_batched_shape_against_oracle():
    """Grouped-query shape: d 1536, 12 query / 2 kv heads x 128, FFN 8960, rope base 1e6,
    256 visual + 48 text tokens, 75% static; 16 streams x 2 layers against the oracle (16
    streams: enough workgroups for the attention kernel with one query tile per wave)."""
    _check_streams(synth.CONFIGS["gqa"].with_layers(2), B=16, n_vis=256, n_txt=48, static_frac=0.75,
                   seed=4, n_new=2)


def test_gqa_32_streams_properties():
    """The grouped-query configuration at its full batch of 32 streams and 28 layers
    (weights drawn on the GPU).  Identical frames: a sparse prefill must reproduce the full
    recompute, whatever is reused.  Bit for bit where the same kernels with the same K splits
    serve: two sparse prefills with different reuse sets (75% and 80% of the visual tokens:
    different row counts, row-tile counts and row blocks per stream) against each other, and
    a prefill that reuses next to nothing against the full recompute.  Between those two
    groups the FFN-down GEMM splits K differently (it chooses the split from the row count),
    so there the agreement is to rounding, amplified over 28 random-init layers."""
    cfg = synth.CONFIGS["gqa"]
    B, n_vis, n_txt = 32, 256, 48
    gm = GpuModel(cfg, seed=5, max_batch=B, max_seq=320, gain_jitter=0.1, gen_device="cuda:0")
    try:
        e0, _, changed = _random_streams(cfg, B, n_vis, n_txt, 0.75, seed=5)
        full = gm.prefill(e0, n_vis, want_hidden=False)
        t_full, _ = gm.decode(B, n_vis + n_txt, 6, full["token"])
        assert np.isfinite(full["logits"]).all()
        nearly = gm.prefill(e0, n_vis, [[b % 7] for b in range(B)], want_hidden=False)   # one token reused
        np.testing.assert_array_equal(nearly["logits"], full["logits"])
        reuse = [np.flatnonzero(~changed[b]).tolist() for b in range(B)]
        same = gm.prefill(e0, n_vis, reuse, want_hidden=False)
        more = [sorted(set(reuse[b]) | set(np.flatnonzero(changed[b])[:13].tolist())) for b in range(B)]
        same2 = gm.prefill(e0, n_vis, more, want_hidden=False)     # 25 row blocks against 28: same K split
        np.testing.assert_array_equal(same2["logits"], same["logits"])
        # (both sides are within 5e-3 of the oracle at this depth, tests/test_gpu_depth.py: the
        # oracle's own bar holds between them)
        np.testing.assert_allclose(same["logits"], full["logits"], atol=2e-2)
        np.testing.assert_allclose(same["attn_mean"], full["attn_mean"], rtol=1e-2, atol=1e-6)
        t_same, _ = gm.decode(B, n_vis + n_txt, 6, same["token"])
        t_same2, _ = gm.decode(B, n_vis + n_txt, 6, same2["token"])
        np.testing.assert_array_equal(t_same2, t_same)
        sure = np.array([margin(full["logits"][b]) > 0.2 for b in range(B)])
        np.testing.assert_array_equal(same["token"][sure], full["token"][sure])
        del t_full
    finally:
        gm.close()


@pytest.mark.parametrize("scene", ["moving_box", "noisy_distractors"])
def test_frame_stream_with_filter_and_layer_adaptive_reuse(scene):
    """(scene "noisy_distractors": the noise-tolerant setting instead, tau = 17/20 on a dim
    scene with +-8 sensor noise, the moving box and three wandering distractors.)
    The streamed configuration: a textured static background with a 48 x 48 px box
    moving 6 px per frame (85-90% of the patches static), task-relevance filter and
    layer-adaptive reuse on, at the 7B layer shape with 3 layers.  Every step runs
    Alg. 1, the layer ratio, the sparse prefill with per-layer reuse counts and two
    decode passes on the GPU, each against the oracle; the statistics the plan of a step
    is made from are the oracle's (no expected value comes from the GPU)."""
    TOL = TOLS["f16"]
    cfg = CFG.with_layers(3)
    n_frames, tau_task = 5, 0.5
    if scene == "moving_box":
        tau = (249, 250)
        frames, touched = synth.moving_box_stream(H, H, n_frames, seed=21), None
    else:
        n_frames, tau = 4, (17, 20)
        frames, touched = synth.noisy_scene_stream(H, H, n_frames, seed=31, patch=PATCH, noise=8)
    wp = synth.projection_matrix(cfg.d_model, PATCH, 22)
    txt = synth.round_bf16(synth.text_embeddings(N_TXT, cfg.d_model, 23))
    emb = [np.concatenate([synth.round_bf16(synth.visual_embeddings(f, PATCH, wp)), txt]) for f in frames]
    om = oracle_model(cfg, seed=5, gain_jitter=0.1)
    gm = GpuModel(cfg, seed=5, max_batch=1, max_seq=320, gain_jitter=0.1)
    try:
        cache = O.new_cache(cfg, 320)
        want = O.dense_forward(om, emb[0], N_VIS, cache)
        got = gm.prefill(emb[0][None], N_VIS)
        assert np.abs(got["logits"][0] - want["logits"]).max() <= TOL
        n_static_seen, varied = [], False
        for t in range(1, n_frames):
            # The oracle's statistics of step t - 1.  A random-init decoder has a flat
            # entropy profile over depth (alpha would be 0 everywhere), so the profile handed
            # to the planner is sharpened with depth, a^l -> (a^l)^(1 + 4 l): entropy then
            # falls with depth, as the method assumes (Sec. 3.4).
            stats = np.stack([want["attn_mean"][l] ** (1.0 + 4.0 * l)
                              for l in range(cfg.n_layers)]).astype(np.float32)
            # a gain that takes the largest cumulative entropy drop to alpha = 0.6, so that
            # the reuse counts differ over depth whatever the random-init profile is
            ent = O.layer_entropy(stats)
            r_cum = np.cumsum([0.0] + [(ent[l - 1] - ent[l]) / ent[l - 1] for l in range(1, len(ent))])
            gain = float(0.6 / r_cum.max()) if r_cum.max() > 1e-6 else 8.0
            p_final, order, per_layer, alpha = O.plan_step(frames[t - 1], frames[t], PATCH, *tau,
                                                           TOP_K, stats, tau_task, gain)
            counts = [len(s) for s in per_layer]
            sel = gm.select(frames[t - 1][None], frames[t][None], PATCH, *tau, TOP_K,
                            stats[:, None], tau_task)
            assert sel["idx"][0] == p_final and sel["order"][0] == order
            g_alpha, g_counts = gm.layer_ratio(stats[:, None], gain, [len(p_final)])
            np.testing.assert_allclose(g_alpha[0], alpha, atol=1e-6)
            for l in range(cfg.n_layers):
                frac = float(np.float32(alpha[l])) * len(p_final)
                assert abs(int(g_counts[0, l]) - counts[l]) <= (0 if abs(frac - round(frac)) > 1e-3 else 1)
            n_static_seen.append(len(O.select_static(frames[t - 1], frames[t], PATCH, *tau, N_VIS)))
            if touched is not None:    # noise alone never makes a patch dynamic at this threshold
                quiet = set(np.flatnonzero(~(touched[t - 1] | touched[t])).tolist())
                raw = gm.select(frames[t - 1][None], frames[t][None], PATCH, *tau, N_VIS)
                assert quiet <= set(raw["idx"][0])
            varied |= len(set(counts)) > 1
            want = O.sparse_forward(om, emb[t], N_VIS, cache, per_layer)
            got = gm.prefill(emb[t][None], N_VIS, [order], [counts])
            alive = ~np.isnan(want["hidden"][:, 0])
            e_h = np.abs(got["hidden"][0][alive] - want["hidden"][alive]).max()
            e_l = np.abs(got["logits"][0] - want["logits"]).max()
            print("\nframe %d: %d static, reuse per layer %s, max-abs hidden %.4g logits %.4g"
                  % (t, n_static_seen[-1], counts, e_h, e_l))
            assert e_h <= TOL and e_l <= TOL
            assert np.all(np.isnan(got["hidden"][0][~alive]))
            np.testing.assert_allclose(got["attn_mean"][:, 0], want["attn_mean"], atol=1e-4, rtol=2e-2)
            if margin(want["logits"]) > 2 * TOL:
                assert int(got["token"][0]) == want["token"]
            toks, logits = O.decode(om, cache, L, want["token"], 2, return_logits=True)
            gt, gl = gm.decode(1, L, 2, [want["token"]])
            assert np.abs(gl[0] - logits).max() <= TOL
            if all(margin(x) > 2 * TOL for x in logits):
                assert gt[0].tolist() == toks
        assert varied                                        # reuse counts did differ over depth
        # the stream is what the configuration says: 85-90% of the patches static
        if scene == "moving_box":
            assert all(0.80 * N_VIS <= n <= 0.95 * N_VIS for n in n_static_seen), n_static_seen
    finally:
        gm.close()


def test_two_views_and_a_chunk_of_action_rows_in_one_pass():
    """The parallel-decoding shape (an action chunk read off ONE pass instead of 7
    sequential decode passes; two camera views): 512 visual tokens from two stacked
    224 x 224 views (the fixed one mostly static, the wrist view not), 32 prompt tokens
    and 56 action placeholder rows (8 actions x 7 dimensions), which are recomputed at
    every step like the prompt.  7B layer shape, 2 layers; the final hidden states of
    the 56 action rows (what an action head would read) against the oracle.  Attention
    stays causal here (shape only)."""
    TOL = TOLS["f16"]
    cfg = CFG.with_layers(2)
    n_vis, n_txt, n_act, k = 512, 32, 56, 100
    L_ = n_vis + n_txt + n_act
    frames = synth.two_view_stream(H, H, 3, seed=41)
    wp = synth.projection_matrix(cfg.d_model, PATCH, 42)
    tail = synth.round_bf16(synth.text_embeddings(n_txt + n_act, cfg.d_model, 43))
    emb = [np.concatenate([synth.round_bf16(synth.visual_embeddings(f, PATCH, wp)), tail]) for f in frames]
    om = oracle_model(cfg, seed=6, gain_jitter=0.1)
    gm = GpuModel(cfg, seed=6, max_batch=1, max_seq=608, gain_jitter=0.1)
    try:
        cache = O.new_cache(cfg, 608)
        want = O.dense_forward(om, emb[0], n_vis, cache)
        got = gm.prefill(emb[0][None], n_vis)
        assert np.abs(got["hidden"][0] - want["hidden"]).max() <= TOL
        for t in (1, 2):
            stats = want["attn_mean"].astype(np.float32)
            p_final, order, _, _ = O.plan_step(frames[t - 1], frames[t], PATCH, 249, 250, k, stats, 0.5, 1.0)
            sel = gm.select(frames[t - 1][None], frames[t][None], PATCH, 249, 250, k, stats[:, None], 0.5)
            assert sel["idx"][0] == p_final and sel["order"][0] == order
            assert 0 < len(p_final) <= k and max(p_final) < n_vis // 2     # all from the fixed view
            want = O.sparse_forward(om, emb[t], n_vis, cache, [order] * cfg.n_layers)
            got = gm.prefill(emb[t][None], n_vis, [order])
            alive = ~np.isnan(want["hidden"][:, 0])
            assert alive[-n_act:].all() and alive.sum() == L_ - len(p_final)
            e_h = np.abs(got["hidden"][0][alive] - want["hidden"][alive]).max()
            e_a = np.abs(got["hidden"][0][-n_act:] - want["hidden"][-n_act:]).max()
            print("\nstep %d: %d reused, max-abs hidden %.4g (action rows %.4g)" % (t, len(p_final), e_h, e_a))
            assert e_h <= TOL
            assert np.all(np.isnan(got["hidden"][0][~alive]))
            np.testing.assert_allclose(got["attn_mean"][:, 0], want["attn_mean"], atol=1e-4, rtol=2e-2)
    finally:
        gm.close()
