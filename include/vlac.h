/*
 * vlac: VLA-Cache sparse prefill for a Llama-style VLA decoder on MI355X (gfx950).
 *
 * C ABI of the library.  One control step of the method (arXiv 2502.02175) is
 *   vlac_select_static   Alg. 1: which visual tokens may reuse last step's K/V
 *   vlac_layer_ratio     Sec. 3.4: how many of them each decoder layer reuses
 *   vlac_sparse_prefill  Alg. 2: decoder pass over the recomputed rows only
 *   vlac_decode_action   Sec. 3.1 / Appendix: KV-cache decode of the other action tokens
 *
 * Conventions
 *  - Every function returns 0 (VLAC_OK) or a negative vlac_status.  Nothing
 *    throws, aborts or prints.  Arguments are validated on the host before any
 *    GPU work is queued; a failed call queues nothing.
 *  - "device" pointers are HIP device memory owned by the caller and only
 *    borrowed for the call; "host" pointers are ordinary memory.  The library
 *    owns only the opaque context (packed weights, workspace).
 *  - Calls are asynchronous on `stream` (a hipStream_t passed as void*; NULL =
 *    the default stream) and must all use the same stream, or be ordered by the
 *    caller.  Calls on one context must not overlap.
 *  - Sequence layout of one stream: [L_v visual tokens in raster order over the
 *    N x N patch grid][L_t text tokens], positions 0 .. L-1, L = L_v + L_t.
 *    Action tokens decoded after the prefill take positions L, L+1, ...
 *  - Index lists are int32.  bf16 means the upper 16 bits of an IEEE fp32.
 */
#ifndef VLAC_H
#define VLAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  VLAC_OK = 0,
  VLAC_E_NULL = -1,   /* a required pointer is NULL */
  VLAC_E_SHAPE = -2,  /* sizes inconsistent with each other or with the model */
  VLAC_E_RANGE = -3,  /* a scalar or an index is out of its allowed range */
  VLAC_E_STATE = -4,  /* call order: weights missing, cache of a stream never filled */
  VLAC_E_HIP = -5,    /* the HIP runtime reported an error (see vlac_last_hip_error) */
  VLAC_E_NOMEM = -6   /* device or host allocation failed */
} vlac_status;

typedef struct vlac_ctx vlac_ctx;

/* Decoder shape (Sec. 3.1; Llama layout: RMSNorm, rotary embedding in the
 * rotate-half pairing, grouped-query attention, SwiGLU feed-forward).
 * Limits: head_dim is 64 or 128; d_model and vocab are multiples of 32, d_ffn of
 * 16; n_q_heads is a multiple of 4 and of n_kv_heads; max_seq is a multiple of
 * 32 and at most 65536; max_batch at most 32767. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_base;
  int32_t max_batch; /* streams (independent environments, each with its own KV cache) */
  int32_t max_seq;   /* cache slots per stream: L + decoded action tokens, rounded up to 32 */
  int32_t operand_dtype; /* VLAC_OPERAND_BF16, VLAC_OPERAND_F16 or VLAC_OPERAND_F16_W8, see below */
} vlac_model_cfg;

/* 16-bit type of the matrix-core operands (weights as stored inside the context,
 * activations, the KV cache); accumulation, the residual stream, softmax and
 * norm statistics are fp32 in both modes.  Weights are always handed over as
 * bf16.  F16 re-encodes them as fp16, which is exact for every bf16 value of
 * magnitude in [2^-14, 65504], and rounds activations 8 times finer than bf16;
 * conversions to fp16 saturate at +-65504. */
enum { VLAC_OPERAND_BF16 = 0, VLAC_OPERAND_F16 = 1, VLAC_OPERAND_F16_W8 = 2 };
/* F16_W8 (beyond the paper: weight-only 8-bit storage, aimed at the decode passes that the
 * method leaves untouched and that are bound by streaming the weights): as F16, but the
 * context keeps every weight matrix as OCP e4m3 codes with one power-of-two scale per
 * output feature (the smallest with max|w_row| / scale <= 448; codes by round to nearest,
 * ties to even; see vlac_quantize_e4m3), and the kernels expand the codes to fp16 in
 * registers, which is exact.  The weights handed over are bf16 as always; the result is
 * that of the F16 mode with the quantised weights.  Launches of 1024 rows or more (batched
 * streams), which are bound by the matrix cores and not by the weights, expand each matrix
 * to fp16 in a workspace of the context before they use it. */

/* One decoder layer, device pointers, bf16, row-major [out_features, in_features]
 * (y = x W^T).  wqkv rows: all query heads, then all key heads, then all value
 * heads.  w_gate_up rows: the gate projection, then the up projection. */
typedef struct {
  const void* wqkv;      /* [(Hq + 2 Hkv) * hd, d] */
  const void* wo;        /* [d, Hq * hd] */
  const void* w_gate_up; /* [2 F, d] */
  const void* w_down;    /* [d, F] */
  const void* g_attn;    /* [d] RMSNorm gain before attention */
  const void* g_ffn;     /* [d] RMSNorm gain before the feed-forward */
} vlac_layer_w;

const char* vlac_status_string(int status);

/* Creates a context on the current HIP device and allocates its workspace.
 * *out is set only on success. */
int vlac_create(const vlac_model_cfg* cfg, vlac_ctx** out);
int vlac_destroy(vlac_ctx* ctx);

/* Last hipError_t seen by this context (0 = none), for VLAC_E_HIP. */
int vlac_last_hip_error(const vlac_ctx* ctx);

/* Copies one layer's weights into the context in the tiled order the matrix
 * cores consume (the caller's buffers may be freed once the stream has run).
 * All layers and the head must be set before any prefill. */
int vlac_set_layer_weights(vlac_ctx* ctx, int layer, const vlac_layer_w* w, void* stream);
/* g_final [d], w_head [vocab, d], embed [vocab, d] (token embedding table used
 * by vlac_decode_action): device, bf16. */
int vlac_set_head_weights(vlac_ctx* ctx, const void* g_final, const void* w_head,
                          const void* embed, void* stream);

/* Bytes of KV cache for max_batch streams.  The cache is one caller-owned device
 * buffer; its internal order (K and V tiled per 32 positions for the matrix
 * cores, K stored after the rotary embedding) is private to the library.
 * It persists across control steps: it is the state Alg. 2 carries from t-1 to t. */
size_t vlac_kv_cache_bytes(const vlac_model_cfg* cfg);

/* How a projection of a batched prefill (Alg. 2 over the rows of many streams: the
 * many-rows GEMM) cuts its work for a given row count; the kernels decide this on the
 * device, this is the same rule for inspection and tests.  out_features x k is the weight
 * matrix, rows the recomputed rows of the launch, max_splits the most K parts the
 * projection may use (1 unless it adds to the residual stream; 1, 2, 3, 4, 6 or 8 parts are
 * considered, values above 8 count as 8; the library passes how many partial-row sets of the
 * call's row capacity its workspace holds: 8 up to 1024 rows, 3 beyond).
 * Results: rows per work item (256, 192 or 128; a work item is 256 features wide), K parts,
 * work items (weight tiles x parts x row blocks).  Needs neither a context nor a GPU.
 * VLAC_E_NULL / VLAC_E_RANGE on null pointers or non-positive sizes. */
int vlac_plan_many_rows_gemm(int out_features, int k, int rows, int max_splits,
                             int* block_rows, int* k_splits, int* work_items);

/* Zero-fills stream b's part of the cache and marks it "never filled": the next
 * prefill of that stream must be a full one.  Must be called once per stream
 * before its first prefill (the kernels read whole 32-position tiles). */
int vlac_reset_stream(vlac_ctx* ctx, int b, void* kv_cache, void* stream);

/* Waits for `stream`, then reports whether any kernel of this context met an
 * index it had to ignore (reuse index outside [0, L_v), count larger than the
 * stride): VLAC_E_RANGE once, then cleared.  Kernels never act on such entries. */
int vlac_check(vlac_ctx* ctx, void* stream);

/* Measurement aid (no part of the method): while a GEMM class is selected, every
 * launch of that class is bracketed by a pair of HIP events on the launch stream.
 * kind = epilogue + 4 * row class; epilogue 0 QKV+rotary+cache write, 1 projection
 * + residual (attention output, FFN down), 2 gate/up + SwiGLU, 3 output head; row
 * class 0: at most 32 rows (decode, head), 1: more (prefill).  kind -1 switches it off.
 * vlac_profile_read waits for the recorded launches and returns their summed
 * elapsed time and their number, then starts counting afresh (at most 2048
 * launches are recorded between reads).  A bracket measures more than the kernel (the
 * markers are queue packets of their own), so every bracket is followed by one more
 * marker, and vlac_profile_read2 also returns the summed time from the closing marker
 * to that one (marker_ms, may be NULL): what a marker costs right behind a marker on
 * the same busy stream. */
int vlac_profile_select(vlac_ctx* ctx, int kind);
int vlac_profile_read(vlac_ctx* ctx, double* total_ms, int* launches);
int vlac_profile_read2(vlac_ctx* ctx, double* total_ms, double* marker_ms, int* launches);
/* What an event bracket adds to the kernel inside it, in microseconds: brackets 40
 * launches of a one-wave kernel that spins on the GPU's constant-rate wall clock for 20 us
 * and stores the time it saw itself run, waits for `stream`, and returns the mean of
 * (bracket - the kernel's own time) over the last 32.  Uses the split-K workspace: call it
 * while nothing else of this context runs. */
int vlac_profile_bracket_cost(vlac_ctx* ctx, void* stream, double* cost_us);

/* The quantiser of VLAC_OPERAND_F16_W8 on its own: w device bf16 [N, K] row-major ->
 * out_codes device uint8 [N, K] (OCP e4m3: 1 sign, 4 exponent bits of bias 7, 3 mantissa
 * bits, subnormals, no infinities) and out_scales device fp32 [N], with
 * w[n, k] ~ value(out_codes[n, k]) * out_scales[n].  Needs no context. */
int vlac_quantize_e4m3(const void* w, int N, int K, uint8_t* out_codes, float* out_scales, void* stream);

/* Alg. 1 (Sec. 3.2 Eq. sim, Eq. topk; Sec. 3.3 Eq. ptask, Eq. pfinal).
 *
 * frame_prev, frame_cur: device uint8 [B, H, W, 3] (frames t-1 and t).  H and W
 * are multiples of `patch`; L_v = (H/patch) * (W/patch) <= 4096; patch <= 64.
 * A patch is static iff cos(P_t, P_{t-1}) >= tau_num / tau_den, tested exactly in
 * integers (0 <= tau_num <= tau_den, 1 <= tau_den < 2^31); two all-zero patches
 * are static, exactly one all-zero patch is not.  Of the static patches the
 * top_k most similar are kept (exact comparison, ties: lower index), 0 <= top_k <= L_v.
 *
 * attn_mean: device fp32 [n_layers, B, L_v], the out_attn_mean of the previous
 * vlac_sparse_prefill (text-to-vision attention, mean over heads and text rows),
 * or NULL to switch the task-relevance filter off.  layer_mask: host bytes
 * [n_layers], non-zero = layer belongs to the set averaged over (NULL = all).
 * The score S is that average (fp32, layers in ascending order).  The
 * L_v - floor(tau_task * L_v) highest-scoring tokens (ties: lower index) are
 * task-relevant and are removed from the reusable set.
 *
 * out_idx   device int32 [B, stride]: P_final, ascending, first out_count[b] valid
 * out_order device int32 [B, stride]: the same set ordered by (S ascending,
 *           index ascending), the order in which layers pick tokens to reuse
 * out_count device int32 [B]
 * out_relevance device fp32 [B, L_v] or NULL: S
 * stride >= top_k. */
int vlac_select_static(vlac_ctx* ctx, const uint8_t* frame_prev, const uint8_t* frame_cur,
                       int B, int H, int W, int patch, int tau_num, int tau_den, int top_k,
                       const float* attn_mean, const uint8_t* layer_mask, float tau_task,
                       int32_t* out_idx, int32_t* out_order, int32_t* out_count,
                       float* out_relevance, int stride, void* stream);

/* vlac_select_static for callers that cannot allocate device memory and cannot hold a
 * context's workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same results bit for bit, but no context: n_layers (of
 * attn_mean, 1..512; ignored when attn_mean is NULL) is passed directly, and the scratch of
 * the three kernels (patch terms, scores, flags: 17 bytes per patch) lives in a fixed array
 * of VLAC_NOALLOC_MAX_PATCHES patches (1.1 MB) that the library's code object places in the
 * memory of every GPU it is loaded on, until the process ends.  The call makes no
 * allocation of any kind; B * L_v beyond the limit returns VLAC_E_RANGE (as do the argument
 * errors of vlac_select_static, with the same statuses), and nothing is queued then.
 * The address of the array on the current device is looked up on the first call on that
 * device (and by vlac_create): make one of the two before capturing a graph.
 * All calls on one GPU share that GPU's array, which keeps the last call's contents (every
 * call overwrites what it reads, nothing has to be cleared): calls that overlap on one GPU,
 * on whatever streams, race; order them. */
#define VLAC_NOALLOC_MAX_PATCHES 65536
int vlac_select_static_noalloc(const uint8_t* frame_prev, const uint8_t* frame_cur, int B, int H,
                               int W, int patch, int tau_num, int tau_den, int top_k,
                               const float* attn_mean, int n_layers, const uint8_t* layer_mask,
                               float tau_task, int32_t* out_idx, int32_t* out_order,
                               int32_t* out_count, float* out_relevance, int stride, void* stream);

/* Front end for the visual tokens (beyond Alg. 1, in its spirit: a token whose K/V are
 * reused at the first decoder layer, Alg. 2, needs no input embedding either).  The
 * embedding of patch i of frame_cur is the fixed linear map
 *   e_i = (pixels_i / 127.5 - 1) . w_proj,
 * pixels_i = the patch as [patch rows][patch cols][3] bytes, w_proj: device bf16
 * [3 patch^2, d_model] row-major (the stand-in for the vision encoder, which the method
 * leaves alone).  It is computed, in fp32, for every patch EXCEPT the first
 * m = min(reuse_count[b], layer_count[b, 0]) entries of reuse_order[b, :] (the rows that
 * vlac_sparse_prefill with the same lists recomputes at layer 0), and written to
 * embeds[b, i, :]; rows of the excepted patches and rows >= L_v are left untouched.
 * reuse_order / reuse_count both NULL: every patch.  layer_count may be NULL.
 * frame_cur: device uint8 [B, H, W, 3]; embeds: device fp32 [B, L, d_model], L >= L_v;
 * H, W multiples of patch, L_v = (H/patch)(W/patch) <= 4096, patch <= 26. */
int vlac_embed_patches(vlac_ctx* ctx, const uint8_t* frame_cur, int B, int H, int W, int patch,
                       const void* w_proj, const int32_t* reuse_order, const int32_t* reuse_count,
                       int stride, const int32_t* layer_count, float* embeds, int L, void* stream);

/* Sec. 3.4, Eq. reuse_ratio: per stream, entropy E^l of attn_mean[l, b, :]
 * normalised over the vision tokens, R^l = (E^{l-1} - E^l) / E^{l-1} (R^1 = 0;
 * 0 when E^{l-1} = 0), alpha^l = clamp(gain_k * sum_{j<=l} R^j, 0, 1), made
 * non-decreasing over l.
 * reuse_count: device int32 [B] (out_count of vlac_select_static) or NULL.
 * out_alpha: device fp32 [B, n_layers].
 * out_layer_count: device int32 [B, n_layers] = floor(alpha^l * reuse_count[b])
 * (fp32 product), or NULL; requires reuse_count. */
int vlac_layer_ratio(vlac_ctx* ctx, const float* attn_mean, int B, int L_v, float gain_k,
                     const int32_t* reuse_count, float* out_alpha, int32_t* out_layer_count,
                     void* stream);

/* Alg. 2 with the appendix's token-reuse mechanism (Eq. KV reuse in Sec. 4.1).
 *
 * embeds: device fp32 [B, L, d], the input embeddings of frame t, L = L_v + L_t.
 * At layer l stream b reuses, untouched, the cached K/V of the first
 * m = min(layer_count[b, l], reuse_count[b]) tokens of reuse_order[b, :] and
 * recomputes all other rows (every text token always): RMSNorm, QKV, rotary
 * embedding at the row's original position, K/V written in place into
 * kv_cache, causal attention of the recomputed queries over the whole mixed
 * cache, output projection, SwiGLU feed-forward.  m is made non-decreasing over
 * l (a reused token has no hidden state to come back from).
 *
 * reuse_order: device int32 [B, stride]; reuse_count: device int32 [B], or both
 * NULL for a full recompute (required for a stream after vlac_reset_stream).
 * Counts above stride are clamped to stride (and reported, see vlac_check).  stride is also
 * what the host knows of the row count (at least B (L - stride) rows are recomputed) when
 * it chooses the kernels of a launch: pass lists no longer than the selection's top_k.
 * Entries outside [0, L_v) and repeated entries are ignored (see vlac_check).
 * layer_count: device int32 [B, n_layers] or NULL (= reuse_count at every layer).
 *
 * out_attn_mean: device fp32 [n_layers, B, L_v] or NULL: this step's
 *   text-to-vision attention statistic, input of the next step's selection.
 * out_hidden: device fp32 [B, L, d] or NULL: hidden state after the final norm of
 *   every row still recomputed at the last layer; other rows are left untouched.
 * out_logits: device fp32 [B, vocab] or NULL: logits of position L-1.
 * out_token: device int32 [B]: greedy first action token (ties: lower id). */
int vlac_sparse_prefill(vlac_ctx* ctx, const float* embeds, int B, int L_v, int L_t,
                        const int32_t* reuse_order, const int32_t* reuse_count, int stride,
                        const int32_t* layer_count, void* kv_cache, float* out_attn_mean,
                        float* out_hidden, float* out_logits, int32_t* out_token, void* stream);

/* Greedy KV-cache decode of n_new further action tokens (Sec. 3.1; Appendix
 * "Token Reuse Mechanism", last paragraph).  first_token: device int32 [B], the
 * out_token of the prefill; it is embedded at position L, its successor at L+1, ...
 * Requires L + n_new <= max_seq.  Cache positions >= L are scratch that the next
 * control step overwrites.
 * out_tokens: device int32 [B, n_new]; out_logits: device fp32 [B, n_new, vocab] or NULL. */
int vlac_decode_action(vlac_ctx* ctx, int B, int L, int n_new, const int32_t* first_token,
                       void* kv_cache, int32_t* out_tokens, float* out_logits, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VLAC_H */
