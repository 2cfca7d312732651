"""GPU-side harness shared by the gpu tests, the smoke check and the benchmark:
a vlac context with seeded random-init weights loaded, and numpy-in / numpy-out
wrappers around the C-ABI calls.  Holds no arithmetic of the method."""
import numpy as np

import synth


class GpuModel:
    def __init__(self, cfg, seed, max_batch, max_seq, gain_jitter=0.1, std=0.02, device="cuda:0",
                 gen_device="cpu", operand="f16", layer_source=None):
        """gen_device="cpu": the shared reference weights (what the oracle sees);
        a GPU device: weights drawn on the GPU, for timing runs only.
        layer_source: l -> dict of bf16 tensors, in place of synth.make_layer (a test that
        hands the same generated tensors to the oracle)."""
        import torch
        import paper_2502_02175_amd as V
        self.V, self.torch, self.cfg, self.device = V, torch, cfg, device
        self.max_batch, self.max_seq = max_batch, max_seq
        self.ccfg = V.ModelCfg(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads,
                               cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.rms_eps, cfg.rope_base,
                               max_batch, max_seq, {"bf16": 0, "f16": 1, "f16w8": 2}[operand])
        self.ctx = V.vlac_create(self.ccfg)
        for l in range(cfg.n_layers):
            src = layer_source(l) if layer_source else synth.make_layer(
                cfg, seed, l, std=std, gain_jitter=gain_jitter, device=gen_device)
            w = {k: v.to(device) for k, v in src.items()}
            V.vlac_set_layer_weights(self.ctx, l, w)
            torch.cuda.synchronize()
        hd = {k: v.to(device) for k, v in
              synth.make_head(cfg, seed, std=std, gain_jitter=gain_jitter, device=gen_device).items()}
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

    def select(self, prev, cur, patch, tau_num, tau_den, top_k, attn_mean=None, tau_task=0.5,
               layer_mask=None):
        """prev/cur: uint8 [B, H, W, 3]; attn_mean: [n_layers, B, L_v] or None.
        Returns dict idx/order (lists per stream), count, relevance."""
        torch, V, dev = self.torch, self.V, self.device
        B, H, W, _ = prev.shape
        L_v = (H // patch) * (W // patch)
        stride = max(top_k, 1)
        idx = torch.full((B, stride), -1, dtype=torch.int32, device=dev)
        order = torch.full((B, stride), -1, dtype=torch.int32, device=dev)
        cnt = torch.zeros(B, dtype=torch.int32, device=dev)
        rel = torch.zeros((B, L_v), device=dev)
        am = None
        if attn_mean is not None:
            am = torch.tensor(np.ascontiguousarray(attn_mean, dtype=np.float32), device=dev)
        V.vlac_select_static(self.ctx, torch.tensor(np.ascontiguousarray(prev), device=dev),
                             torch.tensor(np.ascontiguousarray(cur), device=dev), B, H, W, patch,
                             tau_num, tau_den, top_k, am, layer_mask, tau_task, idx, order, cnt, rel,
                             stride)
        torch.cuda.synchronize()
        c = cnt.cpu().numpy()
        return {"idx": [idx[b, :c[b]].cpu().tolist() for b in range(B)],
                "order": [order[b, :c[b]].cpu().tolist() for b in range(B)],
                "count": c, "relevance": rel.cpu().numpy()}

    def layer_ratio(self, attn_mean, gain_k, reuse_count):
        """attn_mean [n_layers, B, L_v]; returns (alpha [B, n_layers], layer_count [B, n_layers])."""
        torch, V, dev = self.torch, self.V, self.device
        am = torch.tensor(np.ascontiguousarray(attn_mean, dtype=np.float32), device=dev)
        nl, B, L_v = am.shape
        alpha = torch.empty((B, nl), device=dev)
        lc = torch.empty((B, nl), dtype=torch.int32, device=dev)
        rc = torch.tensor(np.asarray(reuse_count, dtype=np.int32), device=dev)
        V.vlac_layer_ratio(self.ctx, am, B, L_v, gain_k, rc, alpha, lc)
        torch.cuda.synchronize()
        return alpha.cpu().numpy(), lc.cpu().numpy()

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
