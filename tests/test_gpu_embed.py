"""GPU parity of vlac_embed_patches (the patch -> embedding projection for the recomputed
patches only) against the oracle, alone and feeding the sparse prefill."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from helpers import GpuModel, oracle_model

pytestmark = pytest.mark.gpu


def run_embed(gm, frames, patch, w_proj, reuse=None, layer_count=None, L=None, fill=-123.0):
    import torch
    V, dev = gm.V, gm.device
    B, H, W, _ = frames.shape
    L_v = (H // patch) * (W // patch)
    L = L or L_v
    out = torch.full((B, L, gm.cfg.d_model), fill, device=dev)
    ro = rc = lc = None
    stride = 1
    if reuse is not None:
        stride = max(1, max(len(r) for r in reuse))
        a = np.zeros((B, stride), dtype=np.int32)
        for b, r in enumerate(reuse):
            a[b, :len(r)] = r
        ro = torch.tensor(a, device=dev)
        rc = torch.tensor([len(r) for r in reuse], dtype=torch.int32, device=dev)
        if layer_count is not None:
            lc = torch.tensor(np.asarray(layer_count, dtype=np.int32), device=dev)
    V.vlac_embed_patches(gm.ctx, torch.tensor(frames, device=dev), B, H, W, patch,
                         torch.tensor(w_proj, device=dev).to(torch.bfloat16), ro, rc, stride, lc, out, L)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("H,W,patch", [(112, 112, 14), (224, 224, 14), (448, 224, 14), (60, 90, 6)])
def test_embed_matches_oracle(H, W, patch):
    cfg = synth.CONFIGS["tiny"]
    gm = GpuModel(cfg, seed=0, max_batch=3, max_seq=640)
    try:
        rng = np.random.default_rng(H + W)
        B, L_v = 3, (H // patch) * (W // patch)
        frames = rng.integers(0, 256, size=(B, H, W, 3), dtype=np.uint8)
        w = synth.round_bf16(synth.projection_matrix(cfg.d_model, patch, 9))
        reuse = [sorted(rng.choice(L_v, size=n, replace=False).tolist()) for n in (0, L_v // 3, L_v)]
        rng.shuffle(reuse[1])
        got = run_embed(gm, frames, patch, w, reuse, L=L_v + 5)
        for b in range(B):
            want = O.embed_patches(frames[b], patch, w, reuse[b])
            keep = ~np.isnan(want[:, 0])
            assert keep.sum() == L_v - len(reuse[b])
            assert not keep.any() or np.abs(got[b, :L_v][keep] - want[keep]).max() <= 1e-5
            assert np.all(got[b, :L_v][~keep] == -123.0)       # skipped rows are not written
            assert np.all(got[b, L_v:] == -123.0)
        # layer counts: only the first layer_count[b][0] entries of the list are skipped
        lc = [[0] * cfg.n_layers, [5] * cfg.n_layers, [L_v] * cfg.n_layers]
        got = run_embed(gm, frames, patch, w, reuse, lc)
        for b in range(B):
            want = O.embed_patches(frames[b], patch, w, reuse[b][:lc[b][0]])
            keep = ~np.isnan(want[:, 0])
            assert not keep.any() or np.abs(got[b][keep] - want[keep]).max() <= 1e-5
            assert np.all(got[b][~keep] == -123.0)
        # no lists: every patch
        got = run_embed(gm, frames, patch, w)
        for b in range(B):
            assert np.abs(got[b] - O.embed_patches(frames[b], patch, w)).max() <= 1e-5
    finally:
        gm.close()


def test_embed_feeds_the_sparse_prefill():
    """Two steps at the tiny configuration: frame -> Alg. 1 -> embeddings of the recomputed
    patches only -> sparse prefill, all on the GPU, against the oracle's chain."""
    import torch
    cfg = synth.CONFIGS["tiny"]
    H, p, n_txt, k = 112, 14, 16, 32
    L_v = (H // p) ** 2
    prev, cur, _ = synth.frame_pair(H, H, p, 16, seed=2)
    w = synth.round_bf16(synth.projection_matrix(cfg.d_model, p, 3))
    txt = synth.round_bf16(synth.text_embeddings(n_txt, cfg.d_model, 4))
    om = oracle_model(cfg, seed=1)
    gm = GpuModel(cfg, seed=1, max_batch=1, max_seq=128)
    try:
        cache = O.new_cache(cfg, 128)
        e0 = np.concatenate([O.embed_patches(prev, p, w), txt])
        want0 = O.dense_forward(om, e0, L_v, cache)
        g0 = np.concatenate([run_embed(gm, prev[None], p, w)[0], txt])
        got0 = gm.prefill(g0[None], L_v)
        assert np.abs(got0["logits"][0] - want0["logits"]).max() <= 2e-2
        reuse = O.select_static(prev, cur, p, 249, 250, k)
        sel = gm.select(prev[None], cur[None], p, 249, 250, k)
        assert sel["idx"][0] == reuse
        e1 = O.embed_patches(cur, p, w, reuse)
        g1 = run_embed(gm, cur[None], p, w, [sel["order"][0]], fill=float("nan"))[0]
        assert np.array_equal(np.isnan(g1[:, 0]), np.isnan(e1[:, 0]))
        want1 = O.sparse_forward(om, np.concatenate([np.nan_to_num(e1), txt]), L_v, cache, [reuse] * cfg.n_layers)
        got1 = gm.prefill(np.concatenate([g1, txt])[None], L_v, [sel["order"][0]])   # NaN rows are never read
        alive = ~np.isnan(want1["hidden"][:, 0])
        assert np.abs(got1["hidden"][0][alive] - want1["hidden"][alive]).max() <= 2e-2
        assert np.abs(got1["logits"][0] - want1["logits"]).max() <= 2e-2
        assert np.isfinite(got1["logits"]).all()
    finally:
        gm.close()
