"""Pins of the oracle's visual-token front end (the patch -> embedding projection for the
recomputed patches only) against closed forms.  CPU only."""
import numpy as np

import synth
from oracle import vlac_oracle as O


def test_embedding_closed_forms():
    rng = np.random.default_rng(0)
    p, d = 4, 6
    dp = 3 * p * p
    w = rng.standard_normal((dp, d))
    frame = np.zeros((2 * p, 3 * p, 3), dtype=np.uint8)
    frame[:p, :p] = 255                        # patch 0: every pixel +1 after scaling
    e = O.embed_patches(frame, p, w)
    np.testing.assert_allclose(e[0], w.sum(axis=0), rtol=1e-12)
    np.testing.assert_allclose(e[1], -w.sum(axis=0), rtol=1e-12)      # all-zero patch: every pixel -1
    # one pixel of one channel differs: the embedding moves by that pixel's weight row
    g = frame.copy()
    g[p + 1, 2 * p + 3, 2] = 51               # patch 5 = (row 1, col 2); (y 1, x 3, ch 2) -> 51/127.5 = 0.4
    k = (1 * p + 3) * 3 + 2
    e2 = O.embed_patches(g, p, w)
    np.testing.assert_allclose(e2[5] - e[5], 0.4 * w[k], rtol=1e-9, atol=1e-12)
    assert np.array_equal(np.delete(e2, 5, axis=0), np.delete(e, 5, axis=0))


def test_embedding_linear_and_skips():
    rng = np.random.default_rng(1)
    H, p, d = 56, 14, 32
    w = synth.projection_matrix(d, p, 3)
    a = rng.integers(0, 256, size=(H, H, 3), dtype=np.uint8)
    b = rng.integers(0, 256, size=(H, H, 3), dtype=np.uint8)
    ea, eb = O.embed_patches(a, p, w), O.embed_patches(b, p, w)
    mid = ((a.astype(np.int64) + b) // 2).astype(np.uint8)
    odd = ((a.astype(np.int64) + b) % 2).astype(np.float64)            # what the integer mean lost
    em = O.embed_patches(mid, p, w)
    corr = np.stack([(synth.patch_pixels((odd * 255).astype(np.uint8), p)[i] / 255.0 / 2 / 127.5) @ w
                     for i in range(16)])
    # affine map: e(mean) = (e(a) + e(b)) / 2 - (lost half units) . W
    np.testing.assert_allclose(em, (ea + eb) / 2 - corr, atol=1e-9)
    skip = [0, 5, 15]
    es = O.embed_patches(a, p, w, skip)
    assert np.all(np.isnan(es[skip])) and np.array_equal(np.delete(es, skip, 0), np.delete(ea, skip, 0))
    # the input generator used for embeddings elsewhere is the same map (fp32 there)
    np.testing.assert_allclose(synth.visual_embeddings(a, p, w), ea, atol=2e-5)
