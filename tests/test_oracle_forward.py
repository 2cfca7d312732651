"""Pins of the oracle's decoder passes (dense, sparse, decode).  CPU only.

dense_forward is pinned to a textbook Llama decoder assembled from torch's own
routines (rms_norm, scaled_dot_product_attention, silu; the rotary embedding as
a complex multiplication) and to closed forms; sparse_forward is pinned to
dense_forward through the special cases in which token reuse is exact
(Alg. 2 / the appendix's claim that the partial cache update is a valid KV
cache); decode is pinned to a dense pass over the extended sequence."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth
from oracle import vlac_oracle as O
from helpers import oracle_model, tiny_inputs

TINY = synth.CONFIGS["tiny"]
GQA_SMALL = synth.ModelCfg(3, 96, 6, 2, 16, 80, 50, rope_base=1.0e6)


def torch_reference(cfg, model, embeds, n_vis):
    """Textbook decoder from torch library routines, fp64."""
    h = torch.tensor(embeds, dtype=torch.float64)
    L = h.shape[0]
    half = cfg.head_dim // 2
    theta = cfg.rope_base ** (-2.0 * torch.arange(half, dtype=torch.float64) / cfg.head_dim)
    rot = torch.polar(torch.ones(L, half, dtype=torch.float64),
                      torch.arange(L, dtype=torch.float64)[:, None] * theta[None])   # e^{i pos theta}

    def rotary(x):  # [L, H, hd]; pair (i, i+half) is one complex number
        z = torch.complex(x[..., :half], x[..., half:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    attn_mean, ks, vs = [], [], []
    for l in range(cfg.n_layers):
        w = {k: torch.tensor(v, dtype=torch.float64) for k, v in model.layer(l).items()}
        xn = F.rms_norm(h, (cfg.d_model,), w["g_attn"], cfg.rms_eps)
        qkv = F.linear(xn, w["wqkv"])
        q, k, v = torch.split(qkv, [cfg.q_dim, cfg.kv_dim, cfg.kv_dim], dim=-1)
        q = rotary(q.view(L, cfg.n_q_heads, cfg.head_dim))
        k = rotary(k.view(L, cfg.n_kv_heads, cfg.head_dim))
        v = v.view(L, cfg.n_kv_heads, cfg.head_dim)
        ks.append(k.numpy()), vs.append(v.numpy())
        g = cfg.n_q_heads // cfg.n_kv_heads
        kk, vv = k.repeat_interleave(g, dim=1), v.repeat_interleave(g, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kk.transpose(0, 1)[None],
                                           vv.transpose(0, 1)[None], is_causal=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(L, -1), w["wo"])
        xn = F.rms_norm(h, (cfg.d_model,), w["g_ffn"], cfg.rms_eps)
        gu = F.linear(xn, w["w_gate_up"])
        h = h + F.linear(F.silu(gu[:, :cfg.d_ffn]) * gu[:, cfg.d_ffn:], w["w_down"])
        # attention statistics: explicit probabilities, text rows x vision keys
        s = torch.einsum("qhd,khd->hqk", q, kk) / cfg.head_dim ** 0.5
        s = s.masked_fill(~torch.ones(L, L, dtype=torch.bool).tril(), float("-inf"))
        attn_mean.append(torch.softmax(s, dim=-1)[:, n_vis:, :n_vis].mean(dim=(0, 1)).numpy())
    hidden = F.rms_norm(h, (cfg.d_model,), torch.tensor(model.head["g_final"]), cfg.rms_eps)
    logits = F.linear(hidden[-1], torch.tensor(model.head["w_head"]))
    return hidden.numpy(), logits.numpy(), np.array(attn_mean), ks, vs


@pytest.mark.parametrize("cfg,n_vis,n_txt", [(TINY, 20, 6), (GQA_SMALL, 9, 5)])
def test_dense_matches_torch_textbook(cfg, n_vis, n_txt):
    # std 0.2 makes attention far from uniform, so a wrong scale or mask shows
    model = oracle_model(cfg, seed=3, gain_jitter=0.2, std=0.2 if cfg is GQA_SMALL else 0.05)
    rng = np.random.default_rng(0)
    emb = rng.standard_normal((n_vis + n_txt, cfg.d_model))
    cache = O.new_cache(cfg, 64)
    got = O.dense_forward(model, emb, n_vis, cache)
    hidden, logits, attn_mean, ks, vs = torch_reference(cfg, model, emb, n_vis)
    np.testing.assert_allclose(got["hidden"], hidden, atol=1e-9)
    np.testing.assert_allclose(got["logits"], logits, atol=1e-9)
    np.testing.assert_allclose(got["attn_mean"], attn_mean, atol=1e-12)
    L = n_vis + n_txt
    for l in range(cfg.n_layers):
        np.testing.assert_allclose(cache[l][0][:L], ks[l], atol=1e-10)
        np.testing.assert_allclose(cache[l][1][:L], vs[l], atol=1e-10)
    assert got["token"] == int(np.argmax(logits))


def test_rope_properties():
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, 2, 64))
    k = rng.standard_normal((1, 2, 64))
    np.testing.assert_array_equal(O.rope(q, [0], 1e4), q)                      # position 0: identity
    for m, n in ((5, 3), (40, 38), (102, 100)):                               # depends on m-n only
        a = (O.rope(q, [m], 1e4) * O.rope(k, [n], 1e4)).sum()
        b = (O.rope(q, [2], 1e4) * O.rope(k, [0], 1e4)).sum()
        assert a == pytest.approx(b, rel=1e-9)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, [17], 1e6)), np.linalg.norm(q), rtol=1e-12)
    # first pair rotates by exactly pos radians (theta_0 = 1): e_0 -> cos, e_{hd/2} -> sin
    e0 = np.zeros((1, 1, 8))
    e0[0, 0, 0] = 1
    r = O.rope(e0, [1], 1e4)[0, 0]
    assert r[0] == pytest.approx(np.cos(1.0)) and r[4] == pytest.approx(np.sin(1.0))
    # last pair rotates by pos * base^(-(hd-2)/hd)
    e3 = np.zeros((1, 1, 8))
    e3[0, 0, 3] = 1
    r = O.rope(e3, [2], 1e4)[0, 0]
    assert r[3] == pytest.approx(np.cos(2 * 1e4 ** (-6 / 8)))


def test_attn_mean_uniform_closed_form():
    """With W_q = W_k = 0 every score is 0, a text row at position p attends
    uniformly over p+1 keys: A_avg[v] = mean over text rows of 1/(p+1)."""
    cfg = TINY
    base = oracle_model(cfg, seed=4)

    def layer(l):
        w = dict(base.layer(l))
        w["wqkv"] = w["wqkv"].copy()
        w["wqkv"][: cfg.q_dim + cfg.kv_dim] = 0
        return w
    model = O.Model(cfg, layer, base.head)
    n_vis, n_txt = 10, 4
    emb = np.random.default_rng(2).standard_normal((n_vis + n_txt, cfg.d_model))
    want = np.mean([1.0 / (p + 1) for p in range(n_vis, n_vis + n_txt)])
    for fwd in (O.dense_forward(model, emb, n_vis),
                O.sparse_forward(model, emb, n_vis, O.new_cache(cfg, 32), [[], []])):
        np.testing.assert_allclose(fwd["attn_mean"], np.full((cfg.n_layers, n_vis), want), rtol=1e-12)
        assert fwd["attn_mean"].sum(axis=1) == pytest.approx(n_vis * want)


# ---------------- sparse_forward against dense_forward ----------------

@pytest.fixture(scope="module")
def tiny():
    prev, cur, redrawn, e_prev, e_cur = tiny_inputs(seed=0)
    model = oracle_model(TINY, seed=0, std=0.05)
    return dict(prev=prev, cur=cur, redrawn=redrawn, e_prev=e_prev, e_cur=e_cur, model=model, n_vis=64)


def filled_cache(t, emb):
    cache = O.new_cache(TINY, 96)
    ref = O.dense_forward(t["model"], emb, t["n_vis"], cache)
    return cache, ref


def test_sparse_empty_reuse_equals_dense(tiny):
    cache, _ = filled_cache(tiny, tiny["e_prev"])
    want_cache = O.new_cache(TINY, 96)
    want = O.dense_forward(tiny["model"], tiny["e_cur"], 64, want_cache)
    got = O.sparse_forward(tiny["model"], tiny["e_cur"], 64, cache, [[], []])
    for key in ("hidden", "logits", "attn_mean"):
        np.testing.assert_allclose(got[key], want[key], atol=1e-10)
    for l in range(2):
        np.testing.assert_allclose(cache[l][0], want_cache[l][0], atol=1e-10)
        np.testing.assert_allclose(cache[l][1], want_cache[l][1], atol=1e-10)


def test_sparse_identical_frames_equals_dense(tiny):
    """Same frame twice: cached K/V are exactly what recomputation would give,
    so any reuse set, nested any way over depth, reproduces the full recompute."""
    cache, want = filled_cache(tiny, tiny["e_cur"])
    reuse = [[3, 7, 11, 40], [3, 7, 11, 40, 41, 42, 63, 0]]
    got = O.sparse_forward(tiny["model"], tiny["e_cur"], 64, cache, reuse)
    alive = np.array([i not in reuse[1] for i in range(80)])
    np.testing.assert_allclose(got["hidden"][alive], want["hidden"][alive], atol=1e-9)
    np.testing.assert_allclose(got["logits"], want["logits"], atol=1e-9)
    np.testing.assert_allclose(got["attn_mean"], want["attn_mean"], atol=1e-12)
    assert np.all(np.isnan(got["hidden"][~alive]))


def test_sparse_suffix_change_is_prefix_caching(tiny):
    """If every changed token comes after every reused token, the reused
    tokens' K/V depend only on unchanged earlier tokens: textbook prefix caching,
    sparse == full recompute exactly."""
    e_new = tiny["e_prev"].copy()
    e_new[30:64] = tiny["e_cur"][30:64]                 # tokens 30.. change
    cache, _ = filled_cache(tiny, tiny["e_prev"])
    want = O.dense_forward(tiny["model"], e_new, 64)
    reuse = [list(range(30)), list(range(30))]
    got = O.sparse_forward(tiny["model"], e_new, 64, cache, reuse)
    np.testing.assert_allclose(got["hidden"][30:], want["hidden"][30:], atol=1e-9)
    np.testing.assert_allclose(got["logits"], want["logits"], atol=1e-9)
    np.testing.assert_allclose(got["attn_mean"], want["attn_mean"], atol=1e-12)
    # and it is an approximation otherwise: reusing a token placed after a changed one differs
    got2 = O.sparse_forward(tiny["model"], e_new, 64, filled_cache(tiny, tiny["e_prev"])[0],
                            [[], [40]])
    assert np.abs(got2["logits"] - want["logits"]).max() > 1e-6


def test_sparse_one_layer_hybrid_input(tiny):
    """One layer: layer-1 K/V depend only on the token's own embedding, so the
    sparse pass on frame t equals a full pass on the hybrid input whose reused
    rows carry frame t-1's embeddings."""
    cfg1 = TINY.with_layers(1)
    model = O.Model(cfg1, tiny["model"]._layer, tiny["model"].head)
    reuse = [i for i in range(64) if not tiny["redrawn"][i]][::2]
    cache = O.new_cache(cfg1, 96)
    O.dense_forward(model, tiny["e_prev"], 64, cache)
    before = [(k.copy(), v.copy()) for k, v in cache]
    got = O.sparse_forward(model, tiny["e_cur"], 64, cache, [reuse])
    hybrid = tiny["e_cur"].copy()
    hybrid[reuse] = tiny["e_prev"][reuse]
    hyb_cache = O.new_cache(cfg1, 96)
    want = O.dense_forward(model, hybrid, 64, hyb_cache)
    alive = np.array([i not in reuse for i in range(80)])
    np.testing.assert_allclose(got["hidden"][alive], want["hidden"][alive], atol=1e-9)
    np.testing.assert_allclose(got["logits"], want["logits"], atol=1e-9)
    # cache rows: reused positions bit-identical to before, others equal the hybrid state's
    np.testing.assert_array_equal(cache[0][0][reuse], before[0][0][reuse])
    np.testing.assert_array_equal(cache[0][1][reuse], before[0][1][reuse])
    np.testing.assert_allclose(cache[0][0][:80], hyb_cache[0][0][:80], atol=1e-10)
    np.testing.assert_allclose(cache[0][1][:80], hyb_cache[0][1][:80], atol=1e-10)


def test_sparse_reuse_order_irrelevant_and_nesting_enforced(tiny):
    a = O.sparse_forward(tiny["model"], tiny["e_cur"], 64, filled_cache(tiny, tiny["e_prev"])[0],
                         [[5, 9, 2], [2, 9, 5, 33]])
    b = O.sparse_forward(tiny["model"], tiny["e_cur"], 64, filled_cache(tiny, tiny["e_prev"])[0],
                         [[9, 2, 5], [33, 5, 2, 9]])
    np.testing.assert_array_equal(a["logits"], b["logits"])
    with pytest.raises(AssertionError):     # a token dropped at layer 1 cannot return at layer 2
        O.sparse_forward(tiny["model"], tiny["e_cur"], 64, filled_cache(tiny, tiny["e_prev"])[0],
                         [[5, 9], [5]])
    with pytest.raises(AssertionError):     # text tokens are never reused
        O.sparse_forward(tiny["model"], tiny["e_cur"], 64, filled_cache(tiny, tiny["e_prev"])[0],
                         [[70], [70]])


def test_sparse_stale_rows_matter(tiny):
    """The approximation is real: with changed frames and reuse, results differ
    from the full recompute, and reused cache rows stay those of frame t-1."""
    cache, _ = filled_cache(tiny, tiny["e_prev"])
    before = [(k.copy(), v.copy()) for k, v in cache]
    reuse = [i for i in range(64) if not tiny["redrawn"][i]][:32]
    got = O.sparse_forward(tiny["model"], tiny["e_cur"], 64, cache, [reuse, reuse])
    want = O.dense_forward(tiny["model"], tiny["e_cur"], 64)
    assert 1e-7 < np.abs(got["logits"] - want["logits"]).max() < 0.5
    for l in range(2):
        np.testing.assert_array_equal(cache[l][0][reuse], before[l][0][reuse])
        np.testing.assert_array_equal(cache[l][1][reuse], before[l][1][reuse])
        rec = [i for i in range(80) if i not in reuse]
        assert np.abs(cache[l][0][rec] - before[l][0][rec]).max() > 0


# ---------------- decode ----------------

@pytest.mark.parametrize("cfg", [TINY, GQA_SMALL])
def test_decode_equals_dense_on_extended_sequence(cfg):
    model = oracle_model(cfg, seed=6, std=0.08)
    n_vis, n_txt, n_new = 12, 5, 3
    L = n_vis + n_txt
    emb = np.random.default_rng(3).standard_normal((L, cfg.d_model))
    cache = O.new_cache(cfg, 32)
    first = O.dense_forward(model, emb, n_vis, cache)["token"]
    toks, logits = O.decode(model, cache, L, first, n_new, return_logits=True)
    seq, prev_tok = emb, first
    for i in range(n_new):
        seq = np.concatenate([seq, model.head["embed"][prev_tok][None]])
        ref = O.dense_forward(model, seq, n_vis)
        np.testing.assert_allclose(logits[i], ref["logits"], atol=1e-9)
        assert toks[i] == ref["token"]
        prev_tok = toks[i]
