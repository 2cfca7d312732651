"""The kernels that copy operand tiles global -> LDS with instructions the compiler does not
see (the two many-rows GEMMs of Alg. 2's recomputed rows, the attention kernel with one query
tile per wave) wait for those copies with hand-counted `s_waitcnt vmcnt(n)`.  libvlac_safe.so
is the same library with every such wait replaced by a wait for everything; it computes the
same values in the same order.  Here both builds run the same prefills, over every
specialisation of those kernels (feature blocks per wave, active row tiles, K steps modulo the
ring sizes, row-block sizes, both head dims), and every output and the whole KV cache must
agree BIT FOR BIT: an LDS read that overtakes its copy shows as a difference, where a
tolerance against the oracle could hide it."""
import os

import numpy as np
import pytest

import synth
import paper_2502_02175_amd as V
from helpers import GpuModel

pytestmark = pytest.mark.gpu
SAFE = os.path.join(os.path.dirname(V.lib_path()), "libvlac_safe.so")

CASES = [
    # name, cfg, streams, visual, text tokens, reused tokens per prefill (per stream: k + 3 (b % 3))
    ("K steps 4 / 11", synth.ModelCfg(2, 256, 4, 4, 64, 688, 256), 6, 120, 24, (0, 10, 37, 61, 88, 110)),
    ("K steps 5 / 4 / 6", synth.ModelCfg(2, 320, 4, 4, 64, 384, 256), 6, 120, 24, (0, 10, 37, 61, 88, 110)),
    ("K steps 6 / 8 / 7", synth.ModelCfg(2, 384, 4, 2, 128, 448, 256), 6, 120, 24, (0, 10, 37, 61, 88, 110)),
    # wide enough for row blocks of 256 and 192 rows, long and many enough for the attention
    # kernel with one query tile per wave (streams with 65 rows or more), head dim 64 and 128
    ("head dim 64, 12 streams x 352", synth.ModelCfg(2, 1024, 16, 4, 64, 2816, 256), 12, 320, 32, (0, 150, 270)),
    ("head dim 128, 22 streams x 352", synth.ModelCfg(2, 1024, 8, 8, 128, 2816, 256), 22, 320, 32, (0, 200, 290)),
]


def run_case(cfg, B, n_vis, n_txt, reuse_counts, seed):
    import torch
    L = n_vis + n_txt
    rng = np.random.default_rng(seed)
    emb = synth.round_bf16(rng.standard_normal((len(reuse_counts) + 1, B, L, cfg.d_model)))
    gm = GpuModel(cfg, seed, max_batch=B, max_seq=(L + 31) // 32 * 32, std=0.05, gen_device="cuda:0")
    outs = []
    try:
        outs.append(gm.prefill(emb[0], n_vis))
        for i, k in enumerate(reuse_counts):
            reuse = [sorted(rng.permutation(n_vis)[:min(n_vis, k + 3 * (b % 3))].tolist()) for b in range(B)]
            if i == len(reuse_counts) - 1:       # one stream with few rows, one with nothing reused
                reuse[0] = list(range(n_vis - 8))
                reuse[1] = []
            outs.append(gm.prefill(emb[i + 1], n_vis, reuse))
        kv = gm.kv.cpu().numpy().copy()
    finally:
        gm.close()
    return outs, kv


@pytest.mark.parametrize("name,cfg,B,n_vis,n_txt,reuse_counts", CASES, ids=[c[0] for c in CASES])
def test_full_waits_change_no_bit(name, cfg, B, n_vis, n_txt, reuse_counts):
    assert os.path.exists(SAFE), "libvlac_safe.so is not built (python -m paper_2502_02175_amd.build)"
    try:
        V.use_library(None)
        ref, kv_ref = run_case(cfg, B, n_vis, n_txt, reuse_counts, seed=17)
        V.use_library(SAFE)
        got, kv_got = run_case(cfg, B, n_vis, n_txt, reuse_counts, seed=17)
    finally:
        V.use_library(None)
    assert np.isfinite(ref[0]["logits"]).all()
    for r, g in zip(ref, got):
        for key in ("logits", "token", "attn_mean", "hidden"):
            np.testing.assert_array_equal(r[key], g[key], err_msg=key)
    np.testing.assert_array_equal(kv_ref, kv_got)
