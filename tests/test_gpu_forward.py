"""GPU parity of vlac_sparse_prefill / vlac_decode_action against the oracle.

Tolerance (bf16 matrix-core operands with fp32 accumulation and an fp32 residual
stream against the fp64 oracle on the same bf16-rounded weights): max-abs 2e-2 on
the final-norm hidden states and the logits; greedy tokens exact (seeds are
chosen with a top-1/top-2 logit margin above 4e-2, which the tests assert)."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from helpers import GpuModel, oracle_model, tiny_inputs

pytestmark = pytest.mark.gpu
TOL = 2e-2
TINY = synth.CONFIGS["tiny"]
GQA_S = synth.ModelCfg(3, 256, 8, 2, 128, 352, 320, rope_base=1.0e6)


def margin(logits):
    s = np.sort(np.asarray(logits, dtype=np.float64))
    return s[-1] - s[-2]


def check(got, want, b=0, alive=None, stats=True):
    if alive is None:
        alive = ~np.isnan(want["hidden"][:, 0])
    err_h = np.abs(got["hidden"][b][alive] - want["hidden"][alive]).max()
    err_l = np.abs(got["logits"][b] - want["logits"]).max()
    assert err_h <= TOL and err_l <= TOL, (err_h, err_l)
    # rows that were reused at the last layer are left untouched (NaN fill of the harness)
    assert np.all(np.isnan(got["hidden"][b][~alive]))
    if stats:
        np.testing.assert_allclose(got["attn_mean"][:, b], want["attn_mean"], atol=2e-4, rtol=2e-2)
    if margin(want["logits"]) > 2 * TOL:
        assert int(got["token"][b]) == want["token"]
    return err_h, err_l


@pytest.fixture(scope="module", params=["f16", "bf16"])
def tiny(request):
    prev, cur, redrawn, e_prev, e_cur = tiny_inputs(seed=0)
    om = oracle_model(TINY, seed=0, std=0.05)
    gm = GpuModel(TINY, seed=0, max_batch=2, max_seq=96, std=0.05, operand=request.param)
    yield dict(prev=prev, cur=cur, redrawn=redrawn, e_prev=e_prev, e_cur=e_cur, om=om, gm=gm)
    gm.close()


def test_tiny_two_steps_and_decode(tiny):
    """The tiny reference configuration: step 1 full, step 2 sparse with the
    oracle's selection (top-k 32 of the 48 static patches), then 4 greedy action tokens."""
    om, gm = tiny["om"], tiny["gm"]
    cache = O.new_cache(TINY, 96)
    want1 = O.dense_forward(om, tiny["e_prev"], 64, cache)
    got1 = gm.prefill(tiny["e_prev"][None], 64)
    check(got1, want1)
    p_final, order, per_layer, alpha = O.plan_step(tiny["prev"], tiny["cur"], 14, 249, 250, 32,
                                                   want1["attn_mean"], 0.5, 2.0)
    counts = [len(s) for s in per_layer]
    want2 = O.sparse_forward(om, tiny["e_cur"], 64, cache, per_layer)
    got2 = gm.prefill(tiny["e_cur"][None], 64, [order], [counts])
    check(got2, want2)
    assert margin(want2["logits"]) > 2 * TOL
    toks, logits = O.decode(om, cache, 80, want2["token"], 3, return_logits=True)
    gt, gl = gm.decode(1, 80, 3, [want2["token"]])
    assert np.abs(gl[0] - logits).max() <= TOL
    assert all(margin(l) > 2 * TOL for l in logits)
    assert gt[0].tolist() == toks


def test_full_reuse_every_layer_and_empty_reuse(tiny):
    om, gm = tiny["om"], tiny["gm"]
    cache = O.new_cache(TINY, 96)
    O.dense_forward(om, tiny["e_prev"], 64, cache)
    gm.prefill(tiny["e_prev"][None], 64)
    reuse = [i for i in range(64) if not tiny["redrawn"][i]][:32]
    want = O.sparse_forward(om, tiny["e_cur"], 64, cache, [reuse, reuse])
    got = gm.prefill(tiny["e_cur"][None], 64, [reuse])            # layer_count NULL: all layers
    check(got, want)
    # empty reuse list == full recompute
    want = O.dense_forward(om, tiny["e_prev"], 64)
    got = gm.prefill(tiny["e_prev"][None], 64, [[]])
    check(got, want)


def test_reuse_list_order_does_not_matter(tiny):
    gm = tiny["gm"]
    gm.prefill(tiny["e_prev"][None], 64)
    a = gm.prefill(tiny["e_cur"][None], 64, [[5, 9, 2, 33]])
    gm.prefill(tiny["e_prev"][None], 64)
    b = gm.prefill(tiny["e_cur"][None], 64, [[33, 2, 9, 5]])
    np.testing.assert_array_equal(a["logits"], b["logits"])       # deterministic, bit for bit
    np.testing.assert_array_equal(a["attn_mean"], b["attn_mean"])


@pytest.mark.parametrize("operand", ["f16", "bf16"])
def test_batched_streams_gqa_ragged(operand):
    """3 streams with different reuse sets (ragged row counts, several row tiles,
    grouped-query heads, head_dim 128, FFN width that needs K padding)."""
    cfg = GQA_S
    om = oracle_model(cfg, seed=7, std=0.05)
    gm = GpuModel(cfg, seed=7, max_batch=3, max_seq=160, std=0.05, operand=operand)
    try:
        rng = np.random.default_rng(1)
        n_vis, n_txt, B = 100, 37, 3
        L = n_vis + n_txt
        e0 = synth.round_bf16(rng.standard_normal((B, L, cfg.d_model)))
        e1 = e0.copy()
        changed = rng.random((B, n_vis)) < 0.3
        e1[:, :n_vis][changed] = synth.round_bf16(rng.standard_normal((int(changed.sum()), cfg.d_model)))
        caches = [O.new_cache(cfg, 160) for _ in range(B)]
        want0 = [O.dense_forward(om, e0[b], n_vis, caches[b]) for b in range(B)]
        got0 = gm.prefill(e0, n_vis)
        for b in range(B):
            check(got0, want0[b], b)
        orders, counts, sets = [], [], []
        for b in range(B):
            static = np.flatnonzero(~changed[b]).tolist()
            rng.shuffle(static)
            if b == 1:
                static = static[:3]
            m = [len(static) // 3, len(static) // 2, len(static)]
            orders.append(static), counts.append(m)
            sets.append([static[:k] for k in m])
        want1 = [O.sparse_forward(om, e1[b], n_vis, caches[b], sets[b]) for b in range(B)]
        got1 = gm.prefill(e1, n_vis, orders, counts)
        for b in range(B):
            check(got1, want1[b], b)
        first = [w["token"] for w in want1]
        gt, gl = gm.decode(B, L, 2, first)
        for b in range(B):
            toks, logits = O.decode(om, caches[b], L, first[b], 2, return_logits=True)
            assert np.abs(gl[b] - logits).max() <= TOL
            if all(margin(l) > 2 * TOL for l in logits):
                assert gt[b].tolist() == toks
    finally:
        gm.close()


def test_long_text_statistic_by_last_arriver():
    """130 text tokens (more than the 96 the deferred reduction of the attention statistic
    provides for): the per-layer reduction by the last workgroup to arrive serves instead.
    Full and sparse step, two streams with different reuse sets."""
    cfg = TINY
    om = oracle_model(cfg, seed=11, std=0.05)
    gm = GpuModel(cfg, seed=11, max_batch=2, max_seq=192, std=0.05)
    try:
        rng = np.random.default_rng(4)
        n_vis, n_txt, B = 40, 130, 2
        e0 = synth.round_bf16(rng.standard_normal((B, n_vis + n_txt, cfg.d_model)))
        e1 = e0.copy()
        e1[:, 5:20] = synth.round_bf16(rng.standard_normal((B, 15, cfg.d_model)))
        caches = [O.new_cache(cfg, 192) for _ in range(B)]
        want0 = [O.dense_forward(om, e0[b], n_vis, caches[b]) for b in range(B)]
        got0 = gm.prefill(e0, n_vis)
        for b in range(B):
            check(got0, want0[b], b)
        reuse = [[0, 1, 2, 3, 4] + list(range(20, 40)), [30, 31, 2]]
        want1 = [O.sparse_forward(om, e1[b], n_vis, caches[b], [reuse[b]] * cfg.n_layers) for b in range(B)]
        for rep in range(3):     # the arrival counters start every launch from zero
            got1 = gm.prefill(e1, n_vis, reuse)
            for b in range(B):
                check(got1, want1[b], b)
    finally:
        gm.close()


def test_many_long_streams_head_dim_64():
    """32 streams of 512 + 32 tokens at the tiny layer shape (head_dim 64): long sequences of
    many streams, where streams with at least 65 rows to recompute take the attention kernel
    with one query tile per wave and the others the one with one query tile per workgroup.
    A third of the streams are 40% static, a third 90%, a third 97% (about 340, 85 and 47 rows)."""
    cfg = TINY
    B, n_vis, n_txt = 32, 512, 32
    L = n_vis + n_txt
    om = oracle_model(cfg, seed=12, std=0.05)
    gm = GpuModel(cfg, seed=12, max_batch=B, max_seq=576, std=0.05)
    try:
        rng = np.random.default_rng(6)
        e0 = synth.round_bf16(rng.standard_normal((B, L, cfg.d_model)))
        e1 = e0.copy()
        frac = np.array([0.4, 0.9, 0.97])[np.arange(B) % 3][:, None]
        changed = rng.random((B, n_vis)) >= frac
        e1[:, :n_vis][changed] = synth.round_bf16(rng.standard_normal((int(changed.sum()), cfg.d_model)))
        caches = [O.new_cache(cfg, 576) for _ in range(B)]
        want0 = [O.dense_forward(om, e0[b], n_vis, caches[b]) for b in range(B)]
        got0 = gm.prefill(e0, n_vis)
        for b in range(B):
            check(got0, want0[b], b)
        reuse = [np.flatnonzero(~changed[b]).tolist() for b in range(B)]
        rows = sorted(L - len(r) for r in reuse)
        assert rows[0] < 65 and 65 <= rows[B // 2] < 128 and rows[-1] > 256
        want1 = [O.sparse_forward(om, e1[b], n_vis, caches[b], [reuse[b]] * cfg.n_layers) for b in range(B)]
        got1 = gm.prefill(e1, n_vis, reuse)
        for b in range(B):
            check(got1, want1[b], b)
    finally:
        gm.close()


def test_mid_size_split_k_with_layer_varying_reuse():
    """d = 1024: the projection GEMMs split K over workgroups and hand partial rows to the
    next row kernel; with reuse counts that grow over depth the row lists of consecutive
    layers differ, so the partial rows must be found through the previous layer's slots.
    Also 6 streams: the decode/head path without the fused norm (more than 4 rows)."""
    cfg = synth.ModelCfg(4, 1024, 8, 8, 128, 2752, 512)
    om = oracle_model(cfg, seed=11, std=0.03)
    gm = GpuModel(cfg, seed=11, max_batch=6, max_seq=128, std=0.03)
    try:
        rng = np.random.default_rng(2)
        n_vis, n_txt, B = 80, 20, 6
        L = n_vis + n_txt
        e0 = synth.round_bf16(rng.standard_normal((B, L, cfg.d_model)))
        e1 = e0.copy()
        changed = rng.random((B, n_vis)) < 0.25
        e1[:, :n_vis][changed] = synth.round_bf16(rng.standard_normal((int(changed.sum()), cfg.d_model)))
        caches = [O.new_cache(cfg, 128) for _ in range(B)]
        for b in range(B):
            O.dense_forward(om, e0[b], n_vis, caches[b])
        gm.prefill(e0, n_vis, want_stats=False, want_hidden=False)
        orders, counts, sets = [], [], []
        for b in range(B):
            static = np.flatnonzero(~changed[b]).tolist()
            rng.shuffle(static)
            n = len(static)
            m = [0, n // 4 + b, n // 2, n] if b % 2 == 0 else [n // 3, n // 3, n - 1, n - 1]
            orders.append(static), counts.append(m)
            sets.append([static[:k] for k in m])
        want = [O.sparse_forward(om, e1[b], n_vis, caches[b], sets[b]) for b in range(B)]
        got = gm.prefill(e1, n_vis, orders, counts)
        for b in range(B):
            check(got, want[b], b)
        first = [w["token"] for w in want]
        gt, gl = gm.decode(B, L, 2, first)
        for b in range(B):
            toks, logits = O.decode(om, caches[b], L, first[b], 2, return_logits=True)
            assert np.abs(gl[b] - logits).max() <= TOL
            if all(margin(l) > 2 * TOL for l in logits):
                assert gt[b].tolist() == toks
    finally:
        gm.close()


def test_row_count_crosses_between_the_two_gemm_kernels_over_depth():
    """Six streams of 80 + 20 tokens at d = 1024 (a capacity of 600 rows: for every GEMM both the
    one-stream and the many-rows kernel are launched and the row count on the device says
    which works).  With reuse counts that grow over depth, layers 0 and 1 recompute more
    than 256 rows, layers 2 and 3 fewer: the partial rows of one kernel's FFN-down GEMM are
    consumed under the other kernel's layer, in the format of the kernel that wrote them."""
    cfg = synth.ModelCfg(4, 1024, 8, 8, 128, 2752, 512)
    om = oracle_model(cfg, seed=15, std=0.03)
    gm = GpuModel(cfg, seed=15, max_batch=6, max_seq=128, std=0.03)
    try:
        rng = np.random.default_rng(3)
        n_vis, n_txt, B = 80, 20, 6
        e0 = synth.round_bf16(rng.standard_normal((B, n_vis + n_txt, cfg.d_model)))
        e1 = e0.copy()
        changed = rng.random((B, n_vis)) < 0.1
        e1[:, :n_vis][changed] = synth.round_bf16(rng.standard_normal((int(changed.sum()), cfg.d_model)))
        caches = [O.new_cache(cfg, 128) for _ in range(B)]
        for b in range(B):
            O.dense_forward(om, e0[b], n_vis, caches[b])
        gm.prefill(e0, n_vis, want_stats=False, want_hidden=False)
        orders, counts, sets = [], [], []
        for b in range(B):
            static = np.flatnonzero(~changed[b]).tolist()
            rng.shuffle(static)
            n = len(static)
            m = [n // 8, n // 2, (7 * n) // 8, n]
            orders.append(static), counts.append(m)
            sets.append([static[:k] for k in m])
        rows = [sum(n_vis + n_txt - counts[b][l] for b in range(B)) for l in range(4)]
        assert rows[0] > 256 and rows[1] > 256 and rows[2] < 256 and rows[3] < 256, rows
        want = [O.sparse_forward(om, e1[b], n_vis, caches[b], sets[b]) for b in range(B)]
        got = gm.prefill(e1, n_vis, orders, counts)
        for b in range(B):
            check(got, want[b], b)
    finally:
        gm.close()


def test_ignored_indices_are_reported(tiny):
    gm = tiny["gm"]
    V, torch = gm.V, gm.torch
    gm.prefill(tiny["e_prev"][None], 64)
    emb = torch.tensor(tiny["e_cur"][None], device="cuda")
    ro = torch.tensor([[3, 3, 70, -1, 8]], dtype=torch.int32, device="cuda")   # repeated, text, negative
    rc = torch.tensor([5], dtype=torch.int32, device="cuda")
    tok = torch.empty(1, dtype=torch.int32, device="cuda")
    logits = torch.empty((1, TINY.vocab), device="cuda")
    V.vlac_sparse_prefill(gm.ctx, emb, 1, 64, 16, ro, rc, 5, None, gm.kv, None, None, logits, tok)
    assert V.vlac_check(gm.ctx, check=False) == -3
    assert V.vlac_check(gm.ctx, check=False) == 0
    torch.cuda.synchronize()
    got = logits.cpu().numpy()[0]
    gm.prefill(tiny["e_prev"][None], 64)
    ref = gm.prefill(tiny["e_cur"][None], 64, [[3, 8]])
    np.testing.assert_array_equal(got, ref["logits"][0])            # only the valid entries acted


def test_state_errors(tiny):
    gm = tiny["gm"]
    V, torch = gm.V, gm.torch
    emb = torch.tensor(tiny["e_cur"][None], device="cuda")
    tok = torch.empty(1, dtype=torch.int32, device="cuda")
    ro = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    rc = torch.zeros(1, dtype=torch.int32, device="cuda")
    V.vlac_reset_stream(gm.ctx, 0, gm.kv)
    st = V.vlac_sparse_prefill(gm.ctx, emb, 1, 64, 16, ro, rc, 4, None, gm.kv, None, None, None, tok,
                               check=False)
    assert st == -4                                                 # reuse on a never-filled cache
    st = V.vlac_decode_action(gm.ctx, 1, 80, 2, tok, gm.kv, torch.empty((1, 2), dtype=torch.int32,
                                                                        device="cuda"), None, check=False)
    assert st == -4
    gm.prefill(tiny["e_prev"][None], 64)
