"""Shared test plumbing: builds oracle models and inputs from the seeded generators."""
import functools

import numpy as np

import synth
from oracle import vlac_oracle as O


def oracle_model(cfg, seed, gain_jitter=0.1, std=0.02, dtype=np.float64, cache_layers=True):
    """Oracle Model over synth weights (bf16 values upcast)."""
    def layer(l):
        return {k: v.float().numpy() for k, v in
                synth.make_layer(cfg, seed, l, std=std, gain_jitter=gain_jitter).items()}
    if cache_layers:
        layer = functools.lru_cache(maxsize=None)(layer)
    head = {k: v.float().numpy() for k, v in
            synth.make_head(cfg, seed, std=std, gain_jitter=gain_jitter).items()}
    return O.Model(cfg, layer, head, dtype=dtype)


def tiny_inputs(seed=0, H=112, patch=14, n_redraw=16, n_text=16, d_model=256, jitter=2):
    """The tiny configuration's inputs: two frames, their visual token embeddings
    (bf16-representable) and the text embeddings."""
    prev, cur, redrawn = synth.frame_pair(H, H, patch, n_redraw, seed, jitter=jitter)
    wp = synth.projection_matrix(d_model, patch, seed + 1)
    txt = synth.round_bf16(synth.text_embeddings(n_text, d_model, seed + 2))
    e_prev = np.concatenate([synth.round_bf16(synth.visual_embeddings(prev, patch, wp)), txt])
    e_cur = np.concatenate([synth.round_bf16(synth.visual_embeddings(cur, patch, wp)), txt])
    return prev, cur, redrawn, e_prev, e_cur


# ---------------------------------------------------------------------------
# GPU side: a context with the synth weights loaded (used by the gpu tests,
# the smoke check and the benchmark).
# ---------------------------------------------------------------------------
class GpuModel:
    def __init__(self, cfg, seed, max_batch, max_seq, gain_jitter=0.1, std=0.02, device="cuda:0"):
        import torch
        import paper_2502_02175_amd as V
        self.V, self.torch, self.cfg, self.device = V, torch, cfg, device
        self.max_batch, self.max_seq = max_batch, max_seq
        self.ccfg = V.ModelCfg(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads,
                               cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.rms_eps, cfg.rope_base,
                               max_batch, max_seq)
        self.ctx = V.vlac_create(self.ccfg)
        for l in range(cfg.n_layers):
            w = {k: v.to(device) for k, v in
                 synth.make_layer(cfg, seed, l, std=std, gain_jitter=gain_jitter).items()}
            V.vlac_set_layer_weights(self.ctx, l, w)
            torch.cuda.synchronize()
        hd = {k: v.to(device) for k, v in
              synth.make_head(cfg, seed, std=std, gain_jitter=gain_jitter).items()}
        V.vlac_set_head_weights(self.ctx, hd["g_final"], hd["w_head"], hd["embed"])
        torch.cuda.synchronize()
        self.kv = torch.empty(V.vlac_kv_cache_bytes(self.ccfg), dtype=torch.uint8, device=device)
        self.kv.fill_(0xFF)  # NaN patterns: the library must not depend on the caller zeroing it
        for b in range(max_batch):
            V.vlac_reset_stream(self.ctx, b, self.kv)

    def prefill(self, embeds, L_v, reuse_order=None, layer_count=None, want_stats=True,
                want_hidden=True):
        """embeds: numpy [B, L, d].  reuse_order: list (per stream) of index lists or None.
        layer_count: [B][n_layers] ints or None.  Returns dict of numpy arrays."""
        torch, V = self.torch, self.V
        dev = self.device
        emb = torch.tensor(np.asarray(embeds, dtype=np.float32), device=dev).contiguous()
        B, L, d = emb.shape
        L_t = L - L_v
        ro = rc = lc = None
        stride = 1
        if reuse_order is not None:
            stride = max(1, max(len(r) for r in reuse_order))
            ro_np = np.zeros((B, stride), dtype=np.int32)
            for b, r in enumerate(reuse_order):
                ro_np[b, :len(r)] = r
            ro = torch.tensor(ro_np, device=dev)
            rc = torch.tensor([len(r) for r in reuse_order], dtype=torch.int32, device=dev)
            if layer_count is not None:
                lc = torch.tensor(np.asarray(layer_count, dtype=np.int32), device=dev).contiguous()
        nl = self.cfg.n_layers
        attn = torch.full((nl, B, max(L_v, 1)), float("nan"), device=dev) if want_stats else None
        hid = torch.full((B, L, d), float("nan"), device=dev) if want_hidden else None
        logits = torch.empty((B, self.cfg.vocab), device=dev)
        tok = torch.empty(B, dtype=torch.int32, device=dev)
        V.vlac_sparse_prefill(self.ctx, emb, B, L_v, L_t, ro, rc, stride, lc, self.kv, attn, hid,
                              logits, tok)
        V.vlac_check(self.ctx)
        torch.cuda.synchronize()
        return {"attn_mean": attn.cpu().numpy() if want_stats else None,
                "hidden": hid.cpu().numpy() if want_hidden else None,
                "logits": logits.cpu().numpy(), "token": tok.cpu().numpy()}

    def decode(self, B, L, n_new, first_token):
        torch, V = self.torch, self.V
        ft = torch.tensor(np.asarray(first_token, dtype=np.int32), device=self.device)
        out = torch.empty((B, n_new), dtype=torch.int32, device=self.device)
        logits = torch.empty((B, n_new, self.cfg.vocab), device=self.device)
        V.vlac_decode_action(self.ctx, B, L, n_new, ft, self.kv, out, logits)
        torch.cuda.synchronize()
        return out.cpu().numpy(), logits.cpu().numpy()

    def close(self):
        if self.ctx:
            self.V.vlac_destroy(self.ctx)
            self.ctx = None
