"""Random-init decoder weights of the benchmark shapes (no trained weights exist here).

Weights are drawn per layer from their own seeded generator, so layer `l` holds
the same values however many layers are built.  All weight matrices are stored
the way the decoder multiplies them, `y = x @ W.T` with W of shape
[out_features, in_features], and are rounded to bf16 so that every consumer
(fp64 oracle, bf16 GPU kernels) sees the same values.
"""
from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class ModelCfg:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    def with_layers(self, n):
        return replace(self, n_layers=n)

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim


CONFIGS = {
    # tiny reference shape: 2 layers, d=256, 4 heads x 64, FFN 688, 256-way head
    "tiny": ModelCfg(2, 256, 4, 4, 64, 688, 256),
    # OpenVLA-7B decoder shape (Llama-2 layout)
    "7b": ModelCfg(32, 4096, 32, 32, 128, 11008, 32000),
    # grouped-query variant: 12 query / 2 kv heads; vocabulary size not fixed by
    # the benchmark description, 32000 is used
    "gqa": ModelCfg(28, 1536, 12, 2, 128, 8960, 32000, rope_base=1.0e6),
}


def round_bf16(x):
    """float array -> float32 array holding bf16-representable values (RNE)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32))
    return t.bfloat16().float().numpy()


def _gen(seed, *tags, device="cpu"):
    g = torch.Generator(device=device)
    g.manual_seed(int(np.random.SeedSequence([seed, *tags]).generate_state(1)[0]))
    return g


def _normal(g, shape, std):
    return (torch.randn(shape, generator=g, dtype=torch.float32, device=g.device) * std).bfloat16()


def make_layer(cfg, seed, layer, std=0.02, gain_jitter=0.0, device="cpu"):
    """bf16 torch tensors of one decoder layer.  With device="cpu" (the default) the
    values are the reference ones every consumer shares; a GPU device draws from that
    device's generator instead (other values, same distribution; for timing runs
    that compare nothing against the CPU).

    wqkv   [(Hq+2Hkv)*hd, d]  rows: all query heads, then key heads, then value heads
    wo     [d, Hq*hd]
    w_gate_up [2F, d]         rows: gate projection, then up projection
    w_down [d, F]
    g_attn, g_ffn [d]         RMSNorm gains (1 + gain_jitter * N(0,1))
    """
    g = _gen(seed, 1, layer, device=device)
    d, F = cfg.d_model, cfg.d_ffn
    out = {
        "wqkv": _normal(g, (cfg.q_dim + 2 * cfg.kv_dim, d), std),
        "wo": _normal(g, (d, cfg.q_dim), std),
        "w_gate_up": _normal(g, (2 * F, d), std),
        "w_down": _normal(g, (d, F), std),
    }
    for name in ("g_attn", "g_ffn"):
        out[name] = (1.0 + gain_jitter * torch.randn(d, generator=g, device=g.device)).bfloat16()
    return out


def make_head(cfg, seed, std=0.02, gain_jitter=0.0, embed_std=1.0, device="cpu"):
    """Final norm gain [d], output head [vocab, d], token embedding table [vocab, d]."""
    g = _gen(seed, 2, device=device)
    d = cfg.d_model
    return {
        "g_final": (1.0 + gain_jitter * torch.randn(d, generator=g, device=g.device)).bfloat16(),
        "w_head": _normal(g, (cfg.vocab, d), std),
        "embed": _normal(g, (cfg.vocab, d), embed_std),
    }
