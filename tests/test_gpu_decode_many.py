"""Decode passes (Sec. 3.1, KV-cache decode of the later action tokens) with more streams
than the few-rows GEMM kernel serves: from 33 streams on a decode pass runs through the
prefill's GEMM and row kernels, which take their rows from a row list.  Every stream's logits
of every decoded token against the oracle."""
import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from helpers import GpuModel, oracle_model

pytestmark = pytest.mark.gpu
TOL = 2e-2


def margin(x):
    s = np.sort(np.asarray(x, dtype=np.float64))
    return s[-1] - s[-2]


@pytest.mark.parametrize("name,cfg,B", [
    ("tiny, 33 streams", synth.CONFIGS["tiny"], 33),
    ("grouped queries, 40 streams", synth.ModelCfg(3, 256, 8, 2, 128, 352, 320, rope_base=1.0e6), 40),
])
def test_decode_with_more_than_32_streams(name, cfg, B):
    n_vis, n_txt, n_new = 48, 11, 3
    L = n_vis + n_txt
    om = oracle_model(cfg, seed=3, std=0.05)
    gm = GpuModel(cfg, seed=3, max_batch=B, max_seq=64, std=0.05)
    try:
        rng = np.random.default_rng(8)
        emb = synth.round_bf16(rng.standard_normal((B, L, cfg.d_model)))
        got = gm.prefill(emb, n_vis)
        caches, first = [], []
        for b in range(B):
            caches.append(O.new_cache(cfg, 64))
            want = O.dense_forward(om, emb[b], n_vis, caches[b])
            assert np.abs(got["logits"][b] - want["logits"]).max() <= TOL
            first.append(want["token"])
        gt, gl = gm.decode(B, L, n_new, first)
        worst, compared = 0.0, 0
        for b in range(B):
            toks, logits = O.decode(om, caches[b], L, first[b], n_new, return_logits=True)
            worst = max(worst, np.abs(gl[b] - logits).max())
            for t in range(n_new):
                if margin(logits[t]) <= 2 * TOL:
                    break
                assert int(gt[b, t]) == toks[t], (b, t)
                compared += 1
        print("\n%s: max-abs logits %.4g over %d decoded tokens, %d compared exactly" %
              (name, worst, B * n_new, compared))
        assert worst <= TOL
        assert compared >= B * n_new // 2
    finally:
        gm.close()
