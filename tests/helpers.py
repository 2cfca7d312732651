"""Shared test plumbing: builds oracle models and inputs from the seeded generators."""
import functools

import numpy as np

import synth
from oracle import vlac_oracle as O


def oracle_model(cfg, seed, gain_jitter=0.1, std=0.02, dtype=np.float64, cache_layers=True, w8=False):
    """Oracle Model over synth weights (bf16 values upcast).  w8: every weight matrix is
    replaced by what weight-only e4m3 storage keeps of it (the oracle's own quantiser)."""
    from oracle import fp8 as Q

    def keep(k, v):
        v = v.float().numpy()
        return Q.quantize_rows(v)[2].astype(np.float32) if w8 and k.startswith("w") else v

    def layer(l):
        return {k: keep(k, v) for k, v in
                synth.make_layer(cfg, seed, l, std=std, gain_jitter=gain_jitter).items()}
    if cache_layers:
        layer = functools.lru_cache(maxsize=None)(layer)
    head = {k: keep(k, v) for k, v in
            synth.make_head(cfg, seed, std=std, gain_jitter=gain_jitter).items()}
    return O.Model(cfg, layer, head, dtype=dtype)


class LayerBank:
    """Generated weights of a deep model, drawn once and handed to both sides: layer l holds
    the tensors of synth.make_layer(cfg, seed, l % distinct) (a decoder of full depth whose
    layers cycle through `distinct` weight sets: drawing and widening 200 M weights takes
    seconds per layer on the host, the depth is what the test is about).  bf16(l): the
    tensors the GPU model packs; f64(l): the same values widened once for the oracle."""

    def __init__(self, cfg, seed, distinct, gain_jitter=0.1, std=0.02):
        self.distinct = min(distinct, cfg.n_layers)
        self._bf16 = [synth.make_layer(cfg, seed, i, std=std, gain_jitter=gain_jitter)
                      for i in range(self.distinct)]
        self._f64 = [None] * self.distinct

    def bf16(self, l):
        return self._bf16[l % self.distinct]

    def f64(self, l):
        i = l % self.distinct
        if self._f64[i] is None:
            self._f64[i] = {k: v.float().numpy().astype(np.float64) for k, v in self._bf16[i].items()}
        return self._f64[i]

    def oracle(self, cfg, seed, gain_jitter=0.1, std=0.02):
        head = {k: v.float().numpy() for k, v in
                synth.make_head(cfg, seed, std=std, gain_jitter=gain_jitter).items()}
        return O.Model(cfg, self.f64, head)


def tiny_inputs(seed=0, H=112, patch=14, n_redraw=16, n_text=16, d_model=256, jitter=2):
    """The tiny configuration's inputs: two frames, their visual token embeddings
    (bf16-representable) and the text embeddings."""
    prev, cur, redrawn = synth.frame_pair(H, H, patch, n_redraw, seed, jitter=jitter)
    wp = synth.projection_matrix(d_model, patch, seed + 1)
    txt = synth.round_bf16(synth.text_embeddings(n_text, d_model, seed + 2))
    e_prev = np.concatenate([synth.round_bf16(synth.visual_embeddings(prev, patch, wp)), txt])
    e_cur = np.concatenate([synth.round_bf16(synth.visual_embeddings(cur, patch, wp)), txt])
    return prev, cur, redrawn, e_prev, e_cur


from harness import GpuModel  # noqa: E402,F401  (GPU-side harness lives at the repo root)
