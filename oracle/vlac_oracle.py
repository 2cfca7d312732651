"""CPU oracle for VLA-Cache (arXiv 2502.02175): TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation of one control step of the
method, written from the paper.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does.  It shares no code
with the HIP library.

Arithmetic: exact Python integers for the patch-similarity test and the top-k
ordering; float64 numpy for the decoder (library matmul / exp / log serve as
steps, no blocking or fusion).  Three decisions that floating point takes for an
integer result are taken in fp32, the precision of the GPU kernels, and say so
where they occur: the relevance ranking, the per-layer reuse count and the
greedy argmax tie rule.

Method passages followed
  Sec. 3.2, Eq. (sim), Eq. (topk), Alg. 1 steps "static token selection"
  Sec. 3.3, Eq. (avistext), Eq. (ptask), Eq. (pfinal), Alg. 1 steps "evict"
  Sec. 3.4, entropy ratio R^l, Eq. (reuse_ratio)
  Alg. 2, Eq. (KV reuse) in Sec. 4.1, Appendix "Token Reuse Mechanism"
  Sec. 3.1 (attention, KV-cache decode)

Readings where the paper is silent or ambiguous are marked "Reading:".

Parity pins: every function here is pinned by tests marked `not gpu`
(closed forms, invariants, brute force, textbook routines of torch) except
`relevant_set`, whose rank-quantile rule is a reading of Eq. (ptask):
"parity unpinned" by the paper for that rule; it is checked by brute force,
by its extremes and by its set-size identity only.
"""
import functools
import math

import numpy as np

# --------------------------------------------------------------------------
# Alg. 1, static token selection (Sec. 3.2)
# --------------------------------------------------------------------------


def patch_terms(frame_prev, frame_cur, patch):
    """Eq. (sim): for every co-located p x p x 3 raw-pixel patch, in raster
    order over the N x N grid, the three exact integers
        dot = P_t . P_{t-1},  na = |P_t|^2,  nb = |P_{t-1}|^2.
    Frames are uint8 [H, W, 3]."""
    H, W, _ = frame_cur.shape
    assert frame_prev.shape == frame_cur.shape and H % patch == 0 and W % patch == 0
    out = []
    for i in range(H // patch):
        for j in range(W // patch):
            a = frame_cur[i * patch:(i + 1) * patch, j * patch:(j + 1) * patch, :]
            b = frame_prev[i * patch:(i + 1) * patch, j * patch:(j + 1) * patch, :]
            a = a.astype(np.int64).ravel()
            b = b.astype(np.int64).ravel()
            out.append((int(a @ b), int(a @ a), int(b @ b)))
    return out


def sim_fraction(dot, na, nb):
    """Sim^2 as an exact fraction (num, den), den > 0.  Pixels are non-negative,
    so Sim >= 0 and ordering by Sim equals ordering by Sim^2.
    Reading: the cosine of Eq. (sim) is undefined for an all-zero patch; two
    all-zero patches count as identical (Sim = 1), exactly one all-zero patch as
    dissimilar (Sim = 0)."""
    if na == 0 and nb == 0:
        return (1, 1)
    if na == 0 or nb == 0:
        return (0, 1)
    return (dot * dot, na * nb)


def is_static(dot, na, nb, tau_num, tau_den):
    """Sim >= tau with tau = tau_num / tau_den, as an integer inequality:
    Sim^2 >= tau^2  <=>  num * tau_den^2 >= tau_num^2 * den."""
    num, den = sim_fraction(dot, na, nb)
    return num * tau_den * tau_den >= tau_num * tau_num * den


def _more_similar_first(x, y):
    """Ordering for Top-k: higher similarity first; equal similarity -> lower
    patch index first (Reading: Eq. (topk) leaves ties open)."""
    (ni, di, i), (nj, dj, j) = x, y
    lhs, rhs = ni * dj, nj * di
    if lhs != rhs:
        return -1 if lhs > rhs else 1
    return -1 if i < j else (1 if i > j else 0)


def select_static(frame_prev, frame_cur, patch, tau_num, tau_den, top_k):
    """Eq. (topk): the `top_k` most similar patches among those with Sim >= tau,
    returned as an ascending list of patch indices.  Fewer than top_k passers:
    all of them."""
    terms = patch_terms(frame_prev, frame_cur, patch)
    passers = []
    for i, (dot, na, nb) in enumerate(terms):
        if is_static(dot, na, nb, tau_num, tau_den):
            num, den = sim_fraction(dot, na, nb)
            passers.append((num, den, i))
    passers.sort(key=functools.cmp_to_key(_more_similar_first))
    return sorted(i for (_, _, i) in passers[:max(top_k, 0)])


# --------------------------------------------------------------------------
# Alg. 1, evicting task-relevant tokens (Sec. 3.3)
# --------------------------------------------------------------------------


def embed_patches(frame, patch, w_proj, skip=()):
    """Front end for the visual tokens, for the patches that are recomputed only (the
    token reuse of Sec. 3.2 / Alg. 2 carried one step further forward: a token whose K/V
    are reused at the first layer needs no embedding).  The embedding is the fixed linear
    map that stands in for the vision encoder: e_i = (pixels_i / 127.5 - 1) . W with
    pixels_i the patch as [rows][cols][channel] bytes and W of shape [3 p^2, d].
    Returns fp64 [n_patches, d]; rows of patches in `skip` are NaN."""
    H, Wd, C = frame.shape
    gh, gw = H // patch, Wd // patch
    w = np.asarray(w_proj, dtype=np.float64)
    out = np.full((gh * gw, w.shape[1]), np.nan)
    skip = set(int(i) for i in skip)
    for r in range(gh):
        for c in range(gw):
            i = r * gw + c
            if i in skip:
                continue
            pix = frame[r * patch:(r + 1) * patch, c * patch:(c + 1) * patch, :].astype(np.float64)
            out[i] = (pix.reshape(-1) / 127.5 - 1.0) @ w
    return out


def task_relevance(attn_mean, layer_mask=None):
    """S_task-relevance: the mean over the selected layers of A^l_avg.

    attn_mean[l, v] is A^l_avg of the previous step: attention probability from
    text queries to vision key v at layer l, averaged over heads and (Reading:
    the paper writes only Mean_heads, a per-token score needs one more mean)
    over the text-query rows.  Reading: Eq. (avistext) slices rows=vision,
    cols=text, which is identically zero under a causal mask with vision first;
    the rows are the text queries and the columns the vision keys.

    The score decides an integer (a ranking), so it is accumulated in fp32 in
    ascending layer order, as the kernel does."""
    a = np.asarray(attn_mean, dtype=np.float32)
    n_layers = a.shape[0]
    sel = [l for l in range(n_layers) if layer_mask is None or layer_mask[l]]
    s = np.zeros(a.shape[1], dtype=np.float32)
    for l in sel:
        s = (s + a[l]).astype(np.float32)
    return (s / np.float32(max(len(sel), 1))).astype(np.float32)


def relevant_set(scores, tau_task):
    """Eq. (ptask).  Reading (rank quantile): the paper ranks the vision tokens
    by score and thresholds; a raw probability threshold of 0.5 could never fire
    for 256 keys, so tau_task is the quantile: the L_v - floor(tau_task * L_v)
    highest-scoring tokens are task-relevant (ties: lower index ranks higher).
    tau_task <= 0: every token is relevant; tau_task >= 1: none."""
    n = len(scores)
    n_rel = n - int(math.floor(float(np.float32(tau_task)) * n))
    n_rel = min(max(n_rel, 0), n)
    order = sorted(range(n), key=lambda v: (-float(scores[v]), v))
    return set(order[:n_rel])


def filter_task_relevant(p_static, scores, tau_task):
    """Eq. (pfinal): P_final = P_static minus P_task-relevant.
    Returns (P_final ascending, reuse_order) where reuse_order lists P_final by
    (score ascending, index ascending): the least relevant tokens first
    (Reading: the layer-adaptive subset keeps the critical tokens recomputed,
    so a partial reuse takes the least relevant ones)."""
    rel = relevant_set(scores, tau_task)
    p_final = [i for i in sorted(p_static) if i not in rel]
    order = sorted(p_final, key=lambda v: (float(scores[v]), v))
    return p_final, order


# --------------------------------------------------------------------------
# Layer-adaptive reuse ratio (Sec. 3.4)
# --------------------------------------------------------------------------


def layer_entropy(attn_mean):
    """E^l: Shannon entropy (natural log) of A^l_avg normalised to a
    distribution over the vision tokens; 0 ln 0 = 0."""
    a = np.asarray(attn_mean, dtype=np.float64)
    ent = np.zeros(a.shape[0])
    for l in range(a.shape[0]):
        tot = a[l].sum()
        if tot <= 0:
            continue
        p = a[l] / tot
        nz = p > 0
        ent[l] = -(p[nz] * np.log(p[nz])).sum()
    return ent


def layer_ratio(attn_mean, gain_k):
    """Eq. (reuse_ratio): alpha^l = min(k * sum_{j<=l} R^j, 1) with
    R^l = (E^{l-1} - E^l) / E^{l-1}.
    Readings: R^1 = 0 (there is no layer 0) and R^l = 0 when E^{l-1} = 0;
    alpha is clamped below at 0 (the sum can be negative); alpha is made
    non-decreasing over depth (running maximum), because a token reused at
    layer l has no hidden state from which layer l+1 could recompute it."""
    ent = layer_entropy(attn_mean)
    alpha = np.zeros(len(ent))
    cum, best = 0.0, 0.0
    for l in range(len(ent)):
        if l > 0 and ent[l - 1] > 0:
            cum += (ent[l - 1] - ent[l]) / ent[l - 1]
        a = min(max(gain_k * cum, 0.0), 1.0)
        best = max(best, a)
        alpha[l] = best
    return alpha


def layer_reuse_counts(alpha, count):
    """Number of tokens of P_final reused at each layer: floor(alpha^l * |P_final|),
    the product taken in fp32 (the kernel's precision, since it decides an integer)."""
    return [int(np.floor(np.float32(a) * np.float32(count))) for a in alpha]


# --------------------------------------------------------------------------
# Decoder math (Sec. 3.1; Llama layout.  Reading: RMSNorm x*rsqrt(mean x^2+eps)*g,
# rotary embedding in the rotate-half pairing (i, i+hd/2) with
# theta_i = base^(-2i/hd), softmax scale 1/sqrt(head_dim), query head h reads
# kv head floor(h * H_kv / H_q), SwiGLU feed-forward.)
# --------------------------------------------------------------------------


class Model:
    """cfg: object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn,
    vocab, rms_eps, rope_base.  layer(l) -> dict of arrays wqkv [(Hq+2Hkv)hd, d],
    wo [d, Hq hd], w_gate_up [2F, d], w_down [d, F], g_attn [d], g_ffn [d];
    head: dict g_final [d], w_head [vocab, d], embed [vocab, d]."""

    def __init__(self, cfg, layer, head, dtype=np.float64):
        self.cfg, self._layer, self.dtype = cfg, layer, dtype
        self.head = {k: np.asarray(v, dtype=dtype) for k, v in head.items()}

    def layer(self, l):
        return {k: np.asarray(v, dtype=self.dtype) for k, v in self._layer(l).items()}


def rmsnorm(x, g, eps):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * g


def rope(x, pos, base):
    """x [rows, heads, hd], pos [rows] (original token positions)."""
    hd = x.shape[-1]
    half = hd // 2
    theta = base ** (-2.0 * np.arange(half) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1).astype(x.dtype)


def silu(x):
    return x / (1.0 + np.exp(-x))


def _softmax(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def _qkv(cfg, w, xn):
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    y = xn @ w["wqkv"].T
    q = y[:, :qd].reshape(-1, cfg.n_q_heads, cfg.head_dim)
    k = y[:, qd:qd + kd].reshape(-1, cfg.n_kv_heads, cfg.head_dim)
    v = y[:, qd + kd:].reshape(-1, cfg.n_kv_heads, cfg.head_dim)
    return q, k, v


def _ffn(cfg, w, xn):
    gu = xn @ w["w_gate_up"].T
    return (silu(gu[:, :cfg.d_ffn]) * gu[:, cfg.d_ffn:]) @ w["w_down"].T


def new_cache(cfg, max_seq, dtype=np.float64):
    """Per layer (K, V), each [max_seq, H_kv, hd]; K is stored after RoPE."""
    shape = (max_seq, cfg.n_kv_heads, cfg.head_dim)
    return [(np.zeros(shape, dtype), np.zeros(shape, dtype)) for _ in range(cfg.n_layers)]


def dense_forward(model, embeds, n_vis, cache=None):
    """Full recompute of one frame: the textbook causal decoder over all L
    tokens ([visual tokens in raster order][text tokens], positions 0..L-1).
    Written with full L x L attention matrices, independently of sparse_forward.

    Returns dict: hidden [L, d] (after the final norm), logits [vocab] of the last
    position, token (greedy), attn_mean [n_layers, n_vis], residual [L, d].
    If `cache` is given, K/V of every position are stored into it."""
    cfg = model.cfg
    h = np.array(embeds, dtype=model.dtype)
    L = h.shape[0]
    pos = np.arange(L)
    group = cfg.n_q_heads // cfg.n_kv_heads
    causal = np.tril(np.ones((L, L), dtype=bool))
    attn_mean = np.zeros((cfg.n_layers, n_vis))
    for l in range(cfg.n_layers):
        w = model.layer(l)
        q, k, v = _qkv(cfg, w, rmsnorm(h, w["g_attn"], cfg.rms_eps))
        q, k = rope(q, pos, cfg.rope_base), rope(k, pos, cfg.rope_base)
        if cache is not None:
            cache[l][0][:L], cache[l][1][:L] = k, v
        out = np.zeros((L, cfg.n_q_heads, cfg.head_dim), dtype=model.dtype)
        for hq in range(cfg.n_q_heads):
            hk = hq // group
            s = q[:, hq] @ k[:, hk].T / math.sqrt(cfg.head_dim)
            p = _softmax(np.where(causal, s, -np.inf))
            out[:, hq] = p @ v[:, hk]
            attn_mean[l] += p[n_vis:, :n_vis].sum(axis=0)
        attn_mean[l] /= cfg.n_q_heads * max(L - n_vis, 1)
        h = h + out.reshape(L, -1) @ w["wo"].T
        h = h + _ffn(cfg, w, rmsnorm(h, w["g_ffn"], cfg.rms_eps))
    return _finish(model, h, attn_mean)


def _finish(model, h, attn_mean):
    hidden = rmsnorm(h, model.head["g_final"], model.cfg.rms_eps)
    logits = hidden[-1] @ model.head["w_head"].T
    return {"hidden": hidden, "logits": logits, "token": greedy(logits),
            "attn_mean": attn_mean, "residual": h}


def greedy(logits):
    """argmax; ties -> lower token id (numpy's argmax rule)."""
    return int(np.argmax(logits))


def sparse_forward(model, embeds, n_vis, cache, reuse_per_layer):
    """Alg. 2 with the Appendix "Token Reuse Mechanism": one prefill in which,
    at layer l, every token i in P_reuse^l keeps K_{t-1}^l(i), V_{t-1}^l(i) as they
    are in `cache` and every other token is recomputed from H_t^l(i):
    RoPE at its ORIGINAL position, its K/V written in place into the cache, and
    its query attends causally over the mixed cache (positions 0..i).

    reuse_per_layer: list (one per layer) of iterables of visual-token indices
    (< n_vis).  Reading: the sets must be nested over depth, a token dropped at
    layer l cannot come back at layer l+1.  Text tokens are always recomputed.

    Returns like dense_forward; `hidden`/`residual` rows of tokens that were
    reused at the last layer are NaN (they have no hidden state).
    `attn_mean` is this step's A^l_avg, the input of the next step's Alg. 1."""
    cfg = model.cfg
    L = embeds.shape[0]
    h = np.array(embeds, dtype=model.dtype)
    alive = np.ones(L, dtype=bool)          # tokens that still carry H_t^l(i)
    group = cfg.n_q_heads // cfg.n_kv_heads
    attn_mean = np.zeros((cfg.n_layers, n_vis))
    for l in range(cfg.n_layers):
        reuse = set(int(i) for i in reuse_per_layer[l])
        assert all(0 <= i < n_vis for i in reuse), "only visual tokens may be reused"
        rows = [i for i in range(L) if i not in reuse]
        assert all(alive[i] for i in rows), "reuse sets must be nested over depth"
        alive[:] = False
        alive[rows] = True
        h[~alive] = np.nan
        rows = np.array(rows)
        w = model.layer(l)
        K, V = cache[l]
        q, k, v = _qkv(cfg, w, rmsnorm(h[rows], w["g_attn"], cfg.rms_eps))
        q, k = rope(q, rows, cfg.rope_base), rope(k, rows, cfg.rope_base)
        K[rows], V[rows] = k, v              # in-place cache update
        out = np.zeros((len(rows), cfg.n_q_heads, cfg.head_dim), dtype=model.dtype)
        for r, i in enumerate(rows):
            for hq in range(cfg.n_q_heads):
                hk = hq // group
                s = K[:i + 1, hk] @ q[r, hq] / math.sqrt(cfg.head_dim)
                p = _softmax(s)
                out[r, hq] = p @ V[:i + 1, hk]
                if i >= n_vis:
                    attn_mean[l] += p[:n_vis]
        attn_mean[l] /= cfg.n_q_heads * max(L - n_vis, 1)
        h[rows] = h[rows] + out.reshape(len(rows), -1) @ w["wo"].T
        h[rows] = h[rows] + _ffn(cfg, w, rmsnorm(h[rows], w["g_ffn"], cfg.rms_eps))
    return _finish(model, h, attn_mean)


def decode(model, cache, L, first_token, n_new, return_logits=False):
    """Standard KV-cache decoding of the remaining action tokens (Sec. 3.1,
    second equation pair; Appendix: later tokens are decoded autoregressively).
    The token produced by the prefill is embedded at position L, and so on;
    each pass appends its K/V to the cache and takes the greedy argmax.
    Returns the n_new tokens (and their logits)."""
    cfg = model.cfg
    group = cfg.n_q_heads // cfg.n_kv_heads
    tokens, all_logits, tok = [], [], int(first_token)
    for step in range(n_new):
        p_ = L + step
        h = np.array(model.head["embed"][tok][None, :], dtype=model.dtype)
        for l in range(cfg.n_layers):
            w = model.layer(l)
            K, V = cache[l]
            q, k, v = _qkv(cfg, w, rmsnorm(h, w["g_attn"], cfg.rms_eps))
            q, k = rope(q, [p_], cfg.rope_base), rope(k, [p_], cfg.rope_base)
            K[p_], V[p_] = k[0], v[0]
            out = np.zeros((1, cfg.n_q_heads, cfg.head_dim), dtype=model.dtype)
            for hq in range(cfg.n_q_heads):
                hk = hq // group
                p = _softmax(K[:p_ + 1, hk] @ q[0, hq] / math.sqrt(cfg.head_dim))
                out[0, hq] = p @ V[:p_ + 1, hk]
            h = h + out.reshape(1, -1) @ w["wo"].T
            h = h + _ffn(cfg, w, rmsnorm(h, w["g_ffn"], cfg.rms_eps))
        logits = rmsnorm(h, model.head["g_final"], cfg.rms_eps)[0] @ model.head["w_head"].T
        tok = greedy(logits)
        tokens.append(tok)
        all_logits.append(logits)
    return (tokens, np.array(all_logits)) if return_logits else tokens


# --------------------------------------------------------------------------
# One whole control step, in the order of Alg. 1 then Alg. 2
# --------------------------------------------------------------------------


def plan_step(frame_prev, frame_cur, patch, tau_num, tau_den, top_k,
              attn_mean_prev, tau_task, gain_k, layer_mask=None):
    """Alg. 1 followed by line 3 of Alg. 2 for one stream.  attn_mean_prev is the
    previous step's A^l_avg (Reading: layer l's own attention is not known before
    its rows are chosen, so the previous step's statistics are used) or None
    (filter off, alpha = 1 at every layer).
    Returns (P_final ascending, reuse_order, per-layer reuse sets, alpha)."""
    p_static = select_static(frame_prev, frame_cur, patch, tau_num, tau_den, top_k)
    if attn_mean_prev is None:
        return p_static, list(p_static), None, None
    scores = task_relevance(attn_mean_prev, layer_mask)
    p_final, order = filter_task_relevant(p_static, scores, tau_task)
    alpha = layer_ratio(attn_mean_prev, gain_k)
    counts = layer_reuse_counts(alpha, len(p_final))
    return p_final, order, [order[:m] for m in counts], alpha
