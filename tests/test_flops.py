"""Pins of the analytic operation counts (host arithmetic): the paper's estimate and
the count of what the kernels compute."""
import numpy as np

import synth
from paper_2502_02175_amd import flops as F

CFG = synth.CONFIGS["7b"]


def test_paper_formula_values_and_identities():
    L, D, M = 288, 4096, 11008
    # Eq. (baseline_layer_flops) written out by hand for the benchmark shape
    assert F.paper_layer_flops(L, D, M) == 4 * 288 * 4096 ** 2 + 2 * 288 ** 2 * 4096 + 2 * 288 * 4096 * 11008
    # reusing nothing saves nothing; reusing everything saves the whole layer
    assert F.paper_layer_saving(0, D, M) == 0
    assert F.paper_layer_saving(L, D, M) == F.paper_layer_flops(L, D, M)
    assert F.paper_selection_overhead(224, 32, 256, D) == 224 ** 2 + 32 * 256 * D + 288 ** 2 * D
    per_layer = [179] * 32
    assert F.paper_step_flops(32, L, per_layer, D, M) == 32 * (F.paper_layer_flops(L, D, M) - F.paper_layer_saving(179, D, M))


def test_true_count_against_a_direct_count():
    """Multiply-adds of a tiny layer counted by brute force (every dot product length)."""
    cfg = synth.ModelCfg(2, 64, 4, 2, 16, 96, 50)
    L = 9
    reused = [[1, 4], [1, 4, 6]]
    want = 0
    for l in range(cfg.n_layers):
        rows = [p for p in range(L) if p not in reused[l]]
        macs = 0
        for p in rows:
            macs += cfg.d_model * (cfg.q_dim + 2 * cfg.kv_dim)        # q, k, v of the row
            macs += cfg.n_q_heads * (p + 1) * cfg.head_dim * 2        # scores and weighted values
            macs += cfg.q_dim * cfg.d_model                           # output projection
            macs += 3 * cfg.d_model * cfg.d_ffn                       # gate, up, down
        want += 2 * macs
    want += 2 * cfg.d_model * cfg.vocab
    assert F.prefill_flops(cfg, L, reused) == want
    # the recomputed-token GEMM work per row and layer that bench.py prices kernels with
    per_row = 2 * (cfg.d_model * (cfg.q_dim + 2 * cfg.kv_dim) + cfg.q_dim * cfg.d_model + 3 * cfg.d_model * cfg.d_ffn)
    dense = F.prefill_flops(cfg, L, [[], []])
    attn = 4 * cfg.q_dim * sum(range(1, L + 1)) * cfg.n_layers
    assert dense == cfg.n_layers * L * per_row + attn + 2 * cfg.d_model * cfg.vocab


def test_7b_shape_magnitudes():
    L = 288
    dense = F.prefill_flops(CFG, L, [[]] * 32)
    # 12.95 GFLOP of GEMM work per token over 32 layers (the figure the roofline uses)
    per_row = 2 * 32 * (4096 * 3 * 4096 + 4096 * 4096 + 3 * 4096 * 11008)
    assert abs(per_row / 1e9 - 12.95) < 0.01
    assert dense > L * per_row and dense < 1.02 * L * per_row + 2 * 4096 * 32000
    sparse = F.prefill_flops(CFG, L, [list(range(179))] * 32)
    assert 0.37 < sparse / dense < 0.39                         # 109 of 288 rows
    assert F.decode_flops(CFG, L, 6) > 6 * per_row
