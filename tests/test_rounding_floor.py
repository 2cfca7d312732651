"""What 16-bit matrix-core operands cost by themselves, on the CPU: the oracle's own
arithmetic (fp64, every sum exact to fp64) with nothing changed but a rounding of each
tensor that the kernels hand to the matrix cores as a 16-bit operand (normed rows, Q, K, V,
the softmax probabilities, the attention output, the SwiGLU output), once to bf16 and once
to fp16, at the 7B layer shape (d 4096, 32 heads x 128, FFN 11008), 3 layers, 96 rows.

This is the floor under any kernel with such operands, whatever its accumulation: the
distance of this pipeline from the unrounded oracle is what the stated tolerance (max-abs
2e-2 on the final-norm hidden states) has to be held against.  It shows that
  * bf16 operands (8 significant bits) cannot meet 2e-2 at this shape with random-init
    weights: rounding alone is already past it after 3 layers, which is why the bf16
    operand mode is tested at 8e-2 there (twice this floor, rounded up);
  * fp16 operands (11 significant bits; exact for the bf16 weights) stay at a quarter of the
    bar (an eighth of the bf16 figure, as 3 more significant bits predict), which is why the
    fp16 operand mode is the default."""
import math

import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O
from helpers import oracle_model

CFG = synth.CONFIGS["7b"].with_layers(3)
L, N_VIS = 96, 64


def round_bf16(x):
    return synth.round_bf16(x).astype(np.float64)


def round_f16(x):
    return np.asarray(x, dtype=np.float16).astype(np.float64)


def forward_with_rounded_operands(om, emb, rnd):
    """dense decoder pass, step by step as O.dense_forward, with `rnd` applied to every
    tensor that is a matrix-core operand in the kernels"""
    cfg = om.cfg
    h = emb.astype(np.float64).copy()
    pos = np.arange(L)
    causal = np.tril(np.ones((L, L), dtype=bool))
    for l in range(cfg.n_layers):
        w = om.layer(l)
        q, k, v = O._qkv(cfg, w, rnd(O.rmsnorm(h, w["g_attn"], cfg.rms_eps)))
        q, k, v = rnd(O.rope(q, pos, cfg.rope_base)), rnd(O.rope(k, pos, cfg.rope_base)), rnd(v)
        out = np.zeros((L, cfg.n_q_heads, cfg.head_dim))
        for hq in range(cfg.n_q_heads):
            s = q[:, hq] @ k[:, hq].T / math.sqrt(cfg.head_dim)
            s = np.where(causal, s, -np.inf)
            e = np.exp(s - s.max(axis=-1, keepdims=True))
            out[:, hq] = (rnd(e) @ v[:, hq]) / e.sum(axis=-1, keepdims=True)   # P is an operand, its sum is fp32
        h = h + rnd(out.reshape(L, -1)) @ w["wo"].T
        gu = rnd(O.rmsnorm(h, w["g_ffn"], cfg.rms_eps)) @ w["w_gate_up"].T
        h = h + rnd(O.silu(gu[:, :cfg.d_ffn]) * gu[:, cfg.d_ffn:]) @ w["w_down"].T
    return O.rmsnorm(h, om.head["g_final"], cfg.rms_eps)


@pytest.fixture(scope="module")
def case():
    om = oracle_model(CFG, seed=0, gain_jitter=0.1)
    emb = synth.round_bf16(np.random.default_rng(0).standard_normal((L, CFG.d_model)))
    want = O.dense_forward(om, emb, N_VIS)["hidden"]
    return om, emb, want


def test_unrounded_emulation_is_the_oracle(case):
    om, emb, want = case
    got = forward_with_rounded_operands(om, emb, lambda x: x)
    assert np.abs(got - want).max() < 1e-9


def test_bf16_operands_alone_exceed_the_stated_tolerance(case):
    om, emb, want = case
    err = np.abs(forward_with_rounded_operands(om, emb, round_bf16) - want).max()
    print("\nbf16 operand rounding alone, 3 layers at the 7B shape: max-abs %.4g" % err)
    assert 2e-2 < err < 4e-2          # past the stated bar, and half of the bf16 mode's test bar


def test_f16_operands_alone_are_far_inside_it(case):
    om, emb, want = case
    err = np.abs(forward_with_rounded_operands(om, emb, round_f16) - want).max()
    print("\nfp16 operand rounding alone, 3 layers at the 7B shape: max-abs %.4g" % err)
    assert err < 1e-2              # (measured 5e-3: a quarter of the bar, an eighth of the bf16 floor)
