"""Analytic operation counts of a control step (host-side arithmetic, no kernels).

Two counts, side by side:
  * the paper's own estimate (Sec. "Theoretical Analysis of Computational Complexity"):
    a layer over L tokens costs about 4 L D^2 + 2 L^2 D + 2 L D M, and reusing L_r tokens
    saves about 4 L_r D^2 + 2 L_r^2 D + 2 L_r D M of it, against a selection overhead of
    about H^2 + L_t L_v D + L^2 D;
  * the count of what the kernels here actually compute for a Llama-layout decoder
    (grouped-query projections, three feed-forward matrices, causal attention of the
    recomputed rows over the whole mixed cache), 2 flops per multiply-add.
"""


def paper_layer_flops(L, D, M):
    """Eq. (baseline_layer_flops): one layer over L tokens."""
    return 4 * L * D * D + 2 * L * L * D + 2 * L * D * M


def paper_layer_saving(L_r, D, M):
    """Eq. (reuse_saving): what reusing L_r tokens saves in one layer."""
    return 4 * L_r * D * D + 2 * L_r * L_r * D + 2 * L_r * D * M


def paper_selection_overhead(H, L_t, L_v, D):
    """The subtrahend of Eq. (final_theoretical_gain): patch similarity, relevance
    filter and entropy estimate, with L = L_v + L_t."""
    L = L_v + L_t
    return H * H + L_t * L_v * D + L * L * D


def paper_step_flops(n_layers, L, reused_per_layer, D, M):
    """The paper's estimate of a prefill: sum over layers of baseline minus saving."""
    return sum(paper_layer_flops(L, D, M) - paper_layer_saving(r, D, M) for r in reused_per_layer[:n_layers])


def layer_flops(d_model, q_dim, kv_dim, d_ffn, rows, key_counts):
    """One decoder layer over `rows` recomputed rows; key_counts: for each such row the
    number of cache positions it attends to (its position + 1)."""
    proj = 2 * rows * d_model * (q_dim + 2 * kv_dim) + 2 * rows * q_dim * d_model
    ffn = 2 * rows * 3 * d_model * d_ffn
    attn = 4 * q_dim * sum(key_counts)          # q.K^T and P.V over every attended key
    return proj + ffn + attn


def prefill_flops(cfg, L, reused_positions_per_layer, vocab_rows=1):
    """cfg: an object with n_layers, d_model, q_dim, kv_dim, d_ffn, vocab.  reused
    positions are given per layer (iterables of positions in [0, L))."""
    total = 0
    for l in range(cfg.n_layers):
        reused = set(reused_positions_per_layer[l])
        keys = [p + 1 for p in range(L) if p not in reused]
        total += layer_flops(cfg.d_model, cfg.q_dim, cfg.kv_dim, cfg.d_ffn, len(keys), keys)
    return total + 2 * vocab_rows * cfg.d_model * cfg.vocab


def decode_flops(cfg, L, n_new):
    """n_new one-row passes over a cache that grows from L positions."""
    total = 0
    for t in range(n_new):
        total += cfg.n_layers * layer_flops(cfg.d_model, cfg.q_dim, cfg.kv_dim, cfg.d_ffn, 1, [L + t + 1])
        total += 2 * cfg.d_model * cfg.vocab
    return total
