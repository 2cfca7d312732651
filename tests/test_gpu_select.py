"""GPU parity of vlac_select_static / vlac_layer_ratio against the oracle.
Index sets are compared bit-exactly (integer work); alpha within 1e-6."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O

pytestmark = pytest.mark.gpu
TINY = synth.CONFIGS["tiny"]


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2502_02175_amd as V
    cfg = V.ModelCfg(4, 256, 4, 4, 64, 688, 256, 1e-6, 1e4, 8, 128, V.OPERAND_F16)
    ctx = V.vlac_create(cfg)
    yield dict(V=V, torch=torch, ctx=ctx, n_layers=4)
    V.vlac_destroy(ctx)


def run_select(gpu, prev, cur, patch, tn, td, k, attn=None, mask=None, tau_task=0.5):
    """prev/cur: uint8 [B, H, W, 3]."""
    V, torch = gpu["V"], gpu["torch"]
    B, H, W, _ = prev.shape
    L_v = (H // patch) * (W // patch)
    stride = max(k, 1)
    dp, dc = torch.tensor(prev, device="cuda"), torch.tensor(cur, device="cuda")
    idx = torch.full((B, stride), -7, dtype=torch.int32, device="cuda")
    order = torch.full((B, stride), -7, dtype=torch.int32, device="cuda")
    cnt = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    rel = torch.zeros((B, L_v), device="cuda")
    da = torch.tensor(attn, device="cuda") if attn is not None else None
    V.vlac_select_static(gpu["ctx"], dp, dc, B, H, W, patch, tn, td, k, da, mask, tau_task,
                         idx, order, cnt, rel, stride)
    torch.cuda.synchronize()
    cnt = cnt.cpu().numpy()
    return ([idx[b, :cnt[b]].cpu().tolist() for b in range(B)],
            [order[b, :cnt[b]].cpu().tolist() for b in range(B)], rel.cpu().numpy())


@pytest.mark.parametrize("H,patch,n_redraw,k", [(112, 14, 16, 32), (112, 14, 16, 64), (224, 14, 77, 180),
                                                (224, 14, 77, 100), (448, 14, 300, 700), (60, 6, 30, 50)])
def test_select_matches_oracle(gpu, H, patch, n_redraw, k):
    B = 3
    prs, cus = [], []
    for b in range(B):
        p, c, _ = synth.frame_pair(H, H, patch, n_redraw, seed=10 * H + b)
        prs.append(p), cus.append(c)
    prev, cur = np.stack(prs), np.stack(cus)
    for tn, td in ((249, 250), (17, 20)):
        idx, order, _ = run_select(gpu, prev, cur, patch, tn, td, k)
        for b in range(B):
            want = O.select_static(prev[b], cur[b], patch, tn, td, k)
            assert idx[b] == want, (H, b, tn)
            assert order[b] == want          # no relevance: reuse order is the index order


@pytest.mark.parametrize("noise,lo,hi", [(8, 16, 80), (20, 8, 64), (2, 32, 224)])
def test_select_on_noisy_streams_with_distractors(gpu, noise, lo, hi):
    """Camera-noise streams with moving distractors at the noise-tolerant threshold
    17/20 and at the simulator's 249/250, with and without the top-k cut and the
    task-relevance filter: index sets and reuse order bit for bit."""
    B, H, p, n_frames, nl = 4, 224, 14, 4, gpu["n_layers"]
    streams = [synth.noisy_scene_stream(H, H, n_frames, seed=90 + b, patch=p, noise=noise, lo=lo, hi=hi,
                                        n_distractors=b)[0] for b in range(B)]
    rng = np.random.default_rng(noise)
    attn = (rng.random((nl, B, 256)) ** 3).astype(np.float32)
    for t in range(1, n_frames):
        prev = np.stack([s[t - 1] for s in streams])
        cur = np.stack([s[t] for s in streams])
        for tn, td in ((17, 20), (249, 250)):
            for k in (100, 256):
                idx, order, _ = run_select(gpu, prev, cur, p, tn, td, k)
                for b in range(B):
                    assert idx[b] == O.select_static(prev[b], cur[b], p, tn, td, k), (t, b, tn, k)
            idx, order, rel = run_select(gpu, prev, cur, p, tn, td, 180, attn, None, 0.4)
            for b in range(B):
                p_static = O.select_static(prev[b], cur[b], p, tn, td, 180)
                want, want_order = O.filter_task_relevant(p_static, O.task_relevance(attn[:, b]), 0.4)
                assert idx[b] == want and order[b] == want_order


def test_select_two_stacked_views(gpu):
    """Two camera views stacked into one 448 x 224 frame (512 patches; H != W): a fixed
    view that is mostly static over a wrist view where next to nothing is."""
    B, H, p = 3, 224, 14
    streams = [synth.two_view_stream(H, H, 4, seed=70 + b) for b in range(B)]
    for t in range(1, 4):
        prev = np.stack([s[t - 1] for s in streams])
        cur = np.stack([s[t] for s in streams])
        for k in (100, 512):
            idx, order, _ = run_select(gpu, prev, cur, p, 249, 250, k)
            for b in range(B):
                assert idx[b] == O.select_static(prev[b], cur[b], p, 249, 250, k)
                assert len(idx[b]) == min(k, len(O.select_static(prev[b], cur[b], p, 249, 250, 512)))


def test_select_ties_zero_patches_and_extremes(gpu):
    rng = np.random.default_rng(3)
    H, p = 56, 14
    f = rng.integers(0, 256, size=(1, H, H, 3), dtype=np.uint8)
    idx, _, _ = run_select(gpu, f, f, p, 249, 250, 5)           # identical frames: all tied
    assert idx[0] == [0, 1, 2, 3, 4]
    idx, _, _ = run_select(gpu, f, f, p, 1, 1, 16)
    assert idx[0] == list(range(16))
    g = f.copy()
    g[0, :14, :14] = 0                                           # black in the current frame only
    g[0, 14:28, :14] = 0
    f2 = f.copy()
    f2[0, 14:28, :14] = 0                                        # black in both frames
    for k in (0, 3, 16):
        idx, _, _ = run_select(gpu, f2, g, p, 249, 250, k)
        assert idx[0] == O.select_static(f2[0], g[0], p, 249, 250, k)
    idx, _, _ = run_select(gpu, f2, g, p, 0, 1, 16)              # tau = 0
    assert idx[0] == list(range(16))
    # near-ties: tiny perturbations of a bright frame give similarities that differ past 1e-12
    base = np.full((1, H, H, 3), 200, dtype=np.uint8)
    cur = base.copy()
    for i in range(16):
        r, c = divmod(i, 4)
        cur[0, r * 14, c * 14, 0] = 200 + (i % 3)               # many exact ties and near ties
    for k in (1, 4, 7, 16):
        idx, _, _ = run_select(gpu, base, cur, p, 249, 250, k)
        assert idx[0] == O.select_static(base[0], cur[0], p, 249, 250, k)


@pytest.mark.parametrize("tau_task", [0.0, 0.2, 0.5, 0.7, 1.0, 1.5])
def test_filter_matches_oracle(gpu, tau_task):
    rng = np.random.default_rng(5)
    B, H, p, k, nl = 2, 112, 14, 40, gpu["n_layers"]
    prs, cus = zip(*[synth.frame_pair(H, H, p, 12, seed=50 + b)[:2] for b in range(B)])
    prev, cur = np.stack(prs), np.stack(cus)
    attn = (rng.random((nl, B, 64)) ** 2).astype(np.float32)
    attn[:, 0, 5] = attn[:, 0, 9]                                # tied scores
    for mask in (None, [1, 0, 1, 0]):
        idx, order, rel = run_select(gpu, prev, cur, p, 249, 250, k, attn, mask, tau_task)
        for b in range(B):
            s = O.task_relevance(attn[:, b], mask)
            np.testing.assert_array_equal(rel[b], s)
            p_static = O.select_static(prev[b], cur[b], p, 249, 250, k)
            want, want_order = O.filter_task_relevant(p_static, s, tau_task)
            assert idx[b] == want and order[b] == want_order


def test_layer_ratio_matches_oracle(gpu):
    V, torch = gpu["V"], gpu["torch"]
    rng = np.random.default_rng(6)
    nl, B, L_v = gpu["n_layers"], 3, 300
    attn = (rng.random((nl, B, L_v)) ** np.arange(1, nl + 1)[:, None, None]).astype(np.float32)
    attn[2, 1] = 0                                               # an all-zero layer: entropy 0
    counts = np.array([100, 0, 77], dtype=np.int32)
    for gain in (0.5, 4.0, 60.0):
        alpha = torch.empty((B, nl), device="cuda")
        lc = torch.empty((B, nl), dtype=torch.int32, device="cuda")
        V.vlac_layer_ratio(gpu["ctx"], torch.tensor(attn, device="cuda"), B, L_v, gain,
                           torch.tensor(counts, device="cuda"), alpha, lc)
        torch.cuda.synchronize()
        alpha, lc = alpha.cpu().numpy(), lc.cpu().numpy()
        for b in range(B):
            want = O.layer_ratio(attn[:, b], gain)
            np.testing.assert_allclose(alpha[b], want, atol=1e-6)
            want_m = O.layer_reuse_counts(want, int(counts[b]))
            for l in range(nl):
                frac = float(np.float32(want[l])) * counts[b]
                if abs(frac - round(frac)) > 1e-3:              # away from a floor boundary: exact
                    assert lc[b, l] == want_m[l]
                else:
                    assert abs(int(lc[b, l]) - want_m[l]) <= 1


@pytest.mark.parametrize("B", [4, 96, 320])
def test_select_with_filter_at_every_launch_shape_of_the_ranking(B):
    """The ranking kernel deals 16, 4 or 1 lanes to a patch by the number of patches in the
    call (here 1024, 24576 and 81920 patches of 224 x 224 frames); the sets and the reuse
    order are integer work and must not depend on that.  The oracle runs on 6 of the streams
    (all of them at B = 4)."""
    import torch
    import paper_2502_02175_amd as V
    H, p, k, nl, L_v = 224, 14, 180, 4, 256
    ctx = V.vlac_create(V.ModelCfg(nl, 256, 4, 4, 64, 688, 256, 1e-6, 1e4, B, 32, V.OPERAND_F16))
    try:
        rng = np.random.default_rng(70 + B)
        pairs = [synth.frame_pair(H, H, p, 40 + 3 * (b % 20), seed=700 + b)[:2] for b in range(min(B, 24))]
        prev = np.stack([pairs[b % len(pairs)][0] for b in range(B)])
        cur = np.stack([pairs[(b * 7 + 3) % len(pairs)][1] if b % 5 == 4 else pairs[b % len(pairs)][1]
                        for b in range(B)])                     # every fifth stream: an unrelated frame pair
        attn = (rng.random((nl, B, L_v)) ** 2).astype(np.float32)
        attn[:, :, 17] = attn[:, :, 200]                         # tied scores in every stream
        idx, order, rel = run_select(dict(V=V, torch=torch, ctx=ctx), prev, cur, p, 249, 250, k, attn, None, 0.6)
        sample = range(B) if B <= 6 else [0, 4, B // 3, B // 2 + 1, B - 2, B - 1]
        for b in sample:
            s = O.task_relevance(attn[:, b], None)
            np.testing.assert_array_equal(rel[b], s)
            want, want_order = O.filter_task_relevant(O.select_static(prev[b], cur[b], p, 249, 250, k), s, 0.6)
            assert idx[b] == want and order[b] == want_order, b
    finally:
        V.vlac_destroy(ctx)


def test_layer_ratio_with_more_layers_than_waves():
    """40 layers on the 16 waves of the ratio kernel's workgroup (layers w, w + 16, w + 32)."""
    import torch
    import paper_2502_02175_amd as V
    nl, B, L_v = 40, 2, 256
    ctx = V.vlac_create(V.ModelCfg(nl, 256, 4, 4, 64, 688, 256, 1e-6, 1e4, B, 32, V.OPERAND_F16))
    try:
        rng = np.random.default_rng(8)
        attn = (rng.random((nl, B, L_v)) ** (1 + 0.2 * np.arange(nl))[:, None, None]).astype(np.float32)
        alpha = torch.empty((B, nl), device="cuda")
        lc = torch.empty((B, nl), dtype=torch.int32, device="cuda")
        V.vlac_layer_ratio(ctx, torch.tensor(attn, device="cuda"), B, L_v, 0.8,
                           torch.tensor(np.array([150, 31], dtype=np.int32), device="cuda"), alpha, lc)
        torch.cuda.synchronize()
        for b in range(B):
            want = O.layer_ratio(attn[:, b], 0.8)
            np.testing.assert_allclose(alpha[b].cpu().numpy(), want, atol=1e-6)
            assert np.all(np.diff(lc[b].cpu().numpy()) >= 0)
    finally:
        V.vlac_destroy(ctx)
