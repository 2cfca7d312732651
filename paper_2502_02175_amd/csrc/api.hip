// C-ABI layer of vlac: argument validation, context and workspace management,
// and the per-step launch sequences.  Semantics of every entry point are stated
// in include/vlac.h.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "common.h"

namespace {

// A kernel that knows how long it ran: one wave reads the constant-rate wall clock (100
// MHz) until `ticks` have passed (or a bounded number of reads, so that it ends whatever
// the clock does) and stores the ticks it saw.  The yardstick for what an event bracket
// adds to the kernel inside it (vlac_profile_bracket_cost).
__global__ void spin_kernel(unsigned long long ticks, unsigned long long* out) {
  const unsigned long long t0 = wall_clock64();
  unsigned long long t = t0;
  for (int it = 0; it < (1 << 20) && t - t0 < ticks; ++it) t = wall_clock64();
  if (threadIdx.x == 0) *out = t - t0;
}

template <class T>
hipError_t dalloc(T** p, size_t n) {
  *p = nullptr;
  return hipMalloc((void**)p, (n ? n : 1) * sizeof(T));
}

size_t frag_elems(int rows, int kpad) { return (size_t)round_up(rows, 32) * kpad; }

size_t kv_elems_per_stream(const vlac_model_cfg& m) {
  return (size_t)m.n_layers * 2 * m.n_kv_heads * m.max_seq * m.head_dim;
}

int check_cfg(const vlac_model_cfg* m) {
  if (m->n_layers < 1 || m->n_layers > 512 || m->d_model < 32 || m->n_q_heads < 1 ||
      m->n_kv_heads < 1 || m->d_ffn < 16 || m->vocab < 32 || m->max_batch < 1 || m->max_seq < 32)
    return VLAC_E_RANGE;
  if (m->head_dim != 64 && m->head_dim != 128) return VLAC_E_SHAPE;
  if (m->d_model % 32 || m->d_ffn % 16 || m->vocab % 32 || m->max_seq % 32) return VLAC_E_SHAPE;
  if (m->n_q_heads % 4 || m->n_q_heads % m->n_kv_heads) return VLAC_E_SHAPE;
  if (m->max_seq > 65536 || m->max_batch > 32767) return VLAC_E_RANGE;
  if (!(m->rms_eps > 0.f) || !(m->rope_base > 1.f)) return VLAC_E_RANGE;
  if (m->operand_dtype != VLAC_OPERAND_BF16 && m->operand_dtype != VLAC_OPERAND_F16 &&
      m->operand_dtype != VLAC_OPERAND_F16_W8)
    return VLAC_E_RANGE;
  return VLAC_OK;
}

void free_all(vlac_ctx* c) {
  if (!c) return;
  if (c->layers) {
    for (int l = 0; l < c->cfg.n_layers; ++l) {
      void* lw[] = {c->layers[l].wqkv, c->layers[l].wo, c->layers[l].wgu,
                    c->layers[l].wdown, c->layers[l].g_attn, c->layers[l].g_ffn,
                    c->layers[l].s_qkv, c->layers[l].s_o, c->layers[l].s_gu, c->layers[l].s_down};
      for (void* p : lw) (void)hipFree(p);
    }
    free(c->layers);
  }
  void* dev[] = {c->w_head, c->s_head, c->scale_tmp, c->wdeq, c->embed, c->g_final, c->rope_cos, c->rope_sin, c->h, c->hdec, c->xa, c->xf,
                 c->qbuf, c->partial, c->rpart, c->counters, c->rows, c->prev_slot, c->n_rows, c->slot_off, c->rank,
                 c->m_layer, c->n_rows_bl, c->statp, c->stat_counters, c->logits, c->tokens,
                 c->dec_rows, c->terms, c->flags, c->embed_list, c->embed_n, c->relevance, c->errword, c->scratch_i,
                 c->zero_tile};
  for (void* p : dev) (void)hipFree(p);
  for (int i = 0; i < c->prof_cap; ++i) {
    if (c->prof_start) (void)hipEventDestroy(c->prof_start[i]);
    if (c->prof_stop) (void)hipEventDestroy(c->prof_stop[i]);
    if (c->prof_mark) (void)hipEventDestroy(c->prof_mark[i]);
  }
  free(c->prof_start); free(c->prof_stop); free(c->prof_mark);
  free(c->layer_set); free(c->filled); free(c->was_reset);
  free(c);
}

}  // namespace

extern "C" {

const char* vlac_status_string(int s) {
  switch (s) {
    case VLAC_OK: return "ok";
    case VLAC_E_NULL: return "required pointer is NULL";
    case VLAC_E_SHAPE: return "inconsistent sizes";
    case VLAC_E_RANGE: return "value out of range";
    case VLAC_E_STATE: return "call order / state";
    case VLAC_E_HIP: return "HIP runtime error";
    case VLAC_E_NOMEM: return "out of memory";
    default: return "unknown status";
  }
}

int vlac_plan_many_rows_gemm(int out_features, int k, int rows, int max_splits,
                             int* block_rows, int* k_splits, int* work_items) {
  if (!block_rows || !k_splits || !work_items) return VLAC_E_NULL;
  if (out_features < 1 || k < 1 || rows < 1 || max_splits < 1) return VLAC_E_RANGE;
  const TallPlan pl = tall_plan(((out_features + 31) / 32 + 7) / 8, rows, max_splits, round_up(k, 64) / 64);
  *block_rows = 64 * pl.rt;
  *k_splits = pl.S;
  *work_items = pl.items();
  return VLAC_OK;
}

size_t vlac_kv_cache_bytes(const vlac_model_cfg* cfg) {
  if (!cfg || check_cfg(cfg) != VLAC_OK) return 0;
  return kv_elems_per_stream(*cfg) * cfg->max_batch * sizeof(bf16_t);
}

int vlac_last_hip_error(const vlac_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int vlac_create(const vlac_model_cfg* cfg, vlac_ctx** out) {
  if (!cfg || !out) return VLAC_E_NULL;
  const int rc = check_cfg(cfg);
  if (rc != VLAC_OK) return rc;
  vlac_ctx* ctx = (vlac_ctx*)calloc(1, sizeof(vlac_ctx));
  if (!ctx) return VLAC_E_NOMEM;
  ctx->cfg = *cfg;
  const vlac_model_cfg& m = ctx->cfg;
  ctx->q_dim = m.n_q_heads * m.head_dim;
  ctx->kv_dim = m.n_kv_heads * m.head_dim;
  ctx->qkv_dim = ctx->q_dim + 2 * ctx->kv_dim;
  ctx->group = m.n_q_heads / m.n_kv_heads;
  ctx->kpad_d = round_up(m.d_model, 64);
  ctx->kpad_q = round_up(ctx->q_dim, 64);
  ctx->kpad_f = round_up(m.d_ffn, 64);
  ctx->max_rows = m.max_batch * m.max_seq;
  ctx->prof_kind = -1;
  ctx->f16 = (m.operand_dtype == VLAC_OPERAND_F16 || m.operand_dtype == VLAC_OPERAND_F16_W8);
  ctx->w8 = (m.operand_dtype == VLAC_OPERAND_F16_W8);
  ctx->layers = (LayerW*)calloc(m.n_layers, sizeof(LayerW));
  ctx->layer_set = (uint8_t*)calloc(m.n_layers, 1);
  ctx->filled = (uint8_t*)calloc(m.max_batch, 1);
  ctx->was_reset = (uint8_t*)calloc(m.max_batch, 1);
  if (!ctx->layers || !ctx->layer_set || !ctx->filled || !ctx->was_reset) {
    free_all(ctx);
    return VLAC_E_NOMEM;
  }
  hipError_t e = hipGetDevice(&ctx->device);
  const int nl = m.n_layers, mb = m.max_batch, ms = m.max_seq, mr = ctx->max_rows;
  const int kpad_x = ctx->kpad_d > ctx->kpad_q ? ctx->kpad_d : ctx->kpad_q;
  ctx->partial_floats = (size_t)64 << 20;  // 256 MiB of split-K workspace
  // partial rows of the projection + residual GEMMs: up to 8 splits of up to 1024 rows
  ctx->rpart_floats = (size_t)8 * (mr < 1024 ? mr : 1024) * m.d_model;
  // (more rows: 3 splits of all rows)
  if (mr >= 1024 && (size_t)3 * mr * m.d_model > ctx->rpart_floats) ctx->rpart_floats = (size_t)3 * mr * m.d_model;
  ctx->n_counters = 1 << 16;
  ctx->stat_tt = ms / 32 + 1;
#define A_(ptr, n) if (e == hipSuccess) e = dalloc(&ctx->ptr, (size_t)(n))
  const int wdiv = ctx->w8 ? 2 : 1;  // e4m3 codes take half the bytes of 16-bit operands
  int max_out = ctx->qkv_dim > 2 * m.d_ffn ? ctx->qkv_dim : 2 * m.d_ffn;
  if (m.vocab > max_out) max_out = m.vocab;
  if (m.d_model > max_out) max_out = m.d_model;
  for (int l = 0; l < nl && e == hipSuccess; ++l) {
    A_(layers[l].wqkv, frag_elems(ctx->qkv_dim, ctx->kpad_d) / wdiv);
    A_(layers[l].wo, frag_elems(m.d_model, ctx->kpad_q) / wdiv);
    A_(layers[l].wgu, frag_elems(2 * m.d_ffn, ctx->kpad_d) / wdiv);
    A_(layers[l].wdown, frag_elems(m.d_model, ctx->kpad_f) / wdiv);
    if (ctx->w8) {
      A_(layers[l].s_qkv, ctx->qkv_dim);
      A_(layers[l].s_o, m.d_model);
      A_(layers[l].s_gu, 2 * m.d_ffn);
      A_(layers[l].s_down, m.d_model);
    }
    A_(layers[l].g_attn, m.d_model);
    A_(layers[l].g_ffn, m.d_model);
  }
  A_(w_head, frag_elems(m.vocab, ctx->kpad_d) / wdiv);
  if (ctx->w8) A_(s_head, m.vocab);
  if (ctx->w8) A_(scale_tmp, max_out);
  if (ctx->w8 && mr >= 1024) {
    // the many-rows GEMM has no variant for e4m3 codes: a launch of 1024 rows or more expands
    // its matrix to fp16 first (the largest of a layer's four fits here)
    size_t most = frag_elems(ctx->qkv_dim, ctx->kpad_d);
    most = std::max(most, frag_elems(m.d_model, ctx->kpad_q));
    most = std::max(most, frag_elems(2 * m.d_ffn, ctx->kpad_d));
    most = std::max(most, frag_elems(m.d_model, ctx->kpad_f));
    A_(wdeq, most);
  }
  A_(embed, (size_t)m.vocab * m.d_model);
  A_(g_final, m.d_model);
  A_(rope_cos, (size_t)ms * (m.head_dim / 2));
  A_(rope_sin, (size_t)ms * (m.head_dim / 2));
  A_(h, (size_t)mr * m.d_model);
  A_(hdec, (size_t)2 * mb * m.d_model);
  A_(xa, frag_elems(mr, kpad_x));
  A_(xf, frag_elems(mr, ctx->kpad_f));
  A_(qbuf, frag_elems(mr, ctx->q_dim));
  A_(partial, ctx->partial_floats);
  A_(rpart, ctx->rpart_floats);
  A_(counters, ctx->n_counters);
  A_(rows, (size_t)(nl + 1) * mr);
  A_(prev_slot, (size_t)nl * mr);
  A_(n_rows, nl + 1);
  A_(slot_off, (size_t)(nl + 1) * (mb + 1));
  A_(rank, (size_t)mr);
  A_(m_layer, (size_t)mb * nl);
  A_(n_rows_bl, (size_t)mb * nl);
  {
    // either one layer's sums for any number of text tiles, or (text of at most 96 tokens)
    // all layers' sums, which one kernel adds up after the last layer
    const size_t one = (size_t)mb * m.n_q_heads * ctx->stat_tt * ms;
    const size_t all = (size_t)nl * mb * m.n_q_heads * kStatDeferTT * ms;
    ctx->statp_floats = one > all ? one : all;
  }
  A_(statp, ctx->statp_floats);
  A_(stat_counters, mb);
  A_(logits, (size_t)mb * m.vocab);
  A_(tokens, mb);
  A_(dec_rows, (size_t)ms * mb + ms + (size_t)ms * (mb + 1));
  A_(terms, (size_t)mb * 4096 * 3);
  A_(flags, (size_t)mb * 4096);
  A_(embed_list, (size_t)mb * 4096);
  A_(embed_n, mb);
  A_(relevance, (size_t)mb * 4096);
  A_(errword, 1);
  A_(zero_tile, 512);
  A_(scratch_i, 64);
#undef A_
  if (e == hipSuccess) e = hipMemset(ctx->counters, 0, ctx->n_counters * sizeof(int));
  if (e == hipSuccess) e = hipMemset(ctx->stat_counters, 0, mb * sizeof(int));
  if (e == hipSuccess) e = hipMemset(ctx->errword, 0, sizeof(int));
  if (e == hipSuccess) e = hipMemset(ctx->zero_tile, 0, 512 * sizeof(bf16_t));
  // operand padding (rows of the last 32-row tile, K padding) must be finite: zero once
  if (e == hipSuccess) e = hipMemset(ctx->xa, 0, frag_elems(mr, kpad_x) * sizeof(bf16_t));
  if (e == hipSuccess) e = hipMemset(ctx->xf, 0, frag_elems(mr, ctx->kpad_f) * sizeof(bf16_t));
  if (e == hipSuccess) e = hipMemset(ctx->qbuf, 0, frag_elems(mr, ctx->q_dim) * sizeof(bf16_t));
  if (e == hipSuccess) {
    // rotary table in fp64 on the host: angle = pos * base^(-2 i / hd)
    const int half = m.head_dim / 2;
    float* hc = (float*)malloc((size_t)ms * half * sizeof(float));
    float* hs = (float*)malloc((size_t)ms * half * sizeof(float));
    if (!hc || !hs) {
      free(hc); free(hs); free_all(ctx);
      return VLAC_E_NOMEM;
    }
    for (int p = 0; p < ms; ++p)
      for (int i = 0; i < half; ++i) {
        const double ang = (double)p * pow((double)m.rope_base, -2.0 * i / m.head_dim);
        hc[(size_t)p * half + i] = (float)cos(ang);
        hs[(size_t)p * half + i] = (float)sin(ang);
      }
    e = hipMemcpy(ctx->rope_cos, hc, (size_t)ms * half * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess)
      e = hipMemcpy(ctx->rope_sin, hs, (size_t)ms * half * sizeof(float), hipMemcpyHostToDevice);
    free(hc); free(hs);
  }
  if (e == hipSuccess) e = (hipError_t)gemm_init();
  if (e == hipSuccess) e = (hipError_t)select_scratch_init();
  if (e != hipSuccess) {
    const bool oom = (e == hipErrorOutOfMemory);
    free_all(ctx);
    (void)hipGetLastError();
    return oom ? VLAC_E_NOMEM : VLAC_E_HIP;
  }
  *out = ctx;
  return VLAC_OK;
}

int vlac_destroy(vlac_ctx* ctx) {
  if (!ctx) return VLAC_E_NULL;
  (void)hipDeviceSynchronize();
  free_all(ctx);
  return VLAC_OK;
}

// Weights [N, K] row-major -> the context's storage (N is a multiple of 32 for every matrix)
static void pack_matrix(vlac_ctx* ctx, const bf16_t* src, int N, int K, bf16_t* dst, float* scales_packed,
                        int kpad, int mode, int p0, int p1, int p2, hipStream_t st) {
  if (ctx->w8) {
    launch_row_scales(src, N, K, ctx->scale_tmp, st);
    launch_pack_e4m3(src, N, K, ctx->scale_tmp, dst, scales_packed, N, kpad, mode, p0, p1, p2, st);
  } else {
    launch_pack(ctx->f16, src, N, K, dst, N, kpad, mode, p0, p1, p2, st);
  }
}

int vlac_quantize_e4m3(const void* w, int N, int K, uint8_t* out_codes, float* out_scales, void* stream) {
  if (!w || !out_codes || !out_scales) return VLAC_E_NULL;
  if (N < 1 || K < 1) return VLAC_E_RANGE;
  launch_row_scales((const bf16_t*)w, N, K, out_scales, (hipStream_t)stream);
  launch_quantize_e4m3((const bf16_t*)w, N, K, out_scales, out_codes, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? VLAC_OK : VLAC_E_HIP;
}

int vlac_set_layer_weights(vlac_ctx* ctx, int layer, const vlac_layer_w* w, void* stream) {
  if (!ctx || !w) return VLAC_E_NULL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return VLAC_E_RANGE;
  if (!w->wqkv || !w->wo || !w->w_gate_up || !w->w_down || !w->g_attn || !w->g_ffn)
    return VLAC_E_NULL;
  const vlac_model_cfg& m = ctx->cfg;
  hipStream_t st = (hipStream_t)stream;
  LayerW& L = ctx->layers[layer];
  pack_matrix(ctx, (const bf16_t*)w->wqkv, ctx->qkv_dim, m.d_model, L.wqkv, L.s_qkv, ctx->kpad_d, 1, ctx->q_dim,
              ctx->kv_dim, m.head_dim, st);
  pack_matrix(ctx, (const bf16_t*)w->wo, m.d_model, ctx->q_dim, L.wo, L.s_o, ctx->kpad_q, 0, 0, 0, 0, st);
  pack_matrix(ctx, (const bf16_t*)w->w_gate_up, 2 * m.d_ffn, m.d_model, L.wgu, L.s_gu, ctx->kpad_d, 2, m.d_ffn, 0,
              0, st);
  pack_matrix(ctx, (const bf16_t*)w->w_down, m.d_model, m.d_ffn, L.wdown, L.s_down, ctx->kpad_f, 0, 0, 0, 0, st);
  launch_bf16_to_f32((const bf16_t*)w->g_attn, L.g_attn, m.d_model, st);
  launch_bf16_to_f32((const bf16_t*)w->g_ffn, L.g_ffn, m.d_model, st);
  VLAC_HIP(hipGetLastError());
  ctx->layer_set[layer] = 1;
  return VLAC_OK;
}

int vlac_set_head_weights(vlac_ctx* ctx, const void* g_final, const void* w_head, const void* embed,
                          void* stream) {
  if (!ctx || !g_final || !w_head || !embed) return VLAC_E_NULL;
  const vlac_model_cfg& m = ctx->cfg;
  hipStream_t st = (hipStream_t)stream;
  pack_matrix(ctx, (const bf16_t*)w_head, m.vocab, m.d_model, ctx->w_head, ctx->s_head, ctx->kpad_d, 0, 0, 0, 0, st);
  launch_bf16_to_f32((const bf16_t*)g_final, ctx->g_final, m.d_model, st);
  VLAC_HIP(hipMemcpyAsync(ctx->embed, embed, (size_t)m.vocab * m.d_model * sizeof(bf16_t),
                          hipMemcpyDeviceToDevice, st));
  VLAC_HIP(hipGetLastError());
  ctx->head_set = true;
  return VLAC_OK;
}

int vlac_reset_stream(vlac_ctx* ctx, int b, void* kv_cache, void* stream) {
  if (!ctx || !kv_cache) return VLAC_E_NULL;
  if (b < 0 || b >= ctx->cfg.max_batch) return VLAC_E_RANGE;
  const size_t bytes = kv_elems_per_stream(ctx->cfg) * sizeof(bf16_t);
  VLAC_HIP(hipMemsetAsync((char*)kv_cache + (size_t)b * bytes, 0, bytes, (hipStream_t)stream));
  ctx->filled[b] = 0;
  ctx->was_reset[b] = 1;
  return VLAC_OK;
}

int vlac_profile_select(vlac_ctx* ctx, int kind) {
  if (!ctx) return VLAC_E_NULL;
  if (kind < -1 || kind >= 8) return VLAC_E_RANGE;
  if (kind >= 0 && !ctx->prof_start) {
    const int cap = 2048;
    ctx->prof_start = (hipEvent_t*)calloc(cap, sizeof(hipEvent_t));
    ctx->prof_stop = (hipEvent_t*)calloc(cap, sizeof(hipEvent_t));
    ctx->prof_mark = (hipEvent_t*)calloc(cap, sizeof(hipEvent_t));
    if (!ctx->prof_start || !ctx->prof_stop || !ctx->prof_mark) return VLAC_E_NOMEM;
    for (int i = 0; i < cap; ++i) {
      VLAC_HIP(hipEventCreate(&ctx->prof_start[i]));
      VLAC_HIP(hipEventCreate(&ctx->prof_stop[i]));
      VLAC_HIP(hipEventCreate(&ctx->prof_mark[i]));
      ctx->prof_cap = i + 1;
    }
  }
  ctx->prof_kind = kind;
  ctx->prof_n = 0;
  return VLAC_OK;
}

int vlac_profile_read2(vlac_ctx* ctx, double* total_ms, double* marker_ms, int* launches) {
  if (!ctx || !total_ms || !launches) return VLAC_E_NULL;
  double tot = 0, mark = 0;
  for (int i = 0; i < ctx->prof_n; ++i) {
    VLAC_HIP(hipEventSynchronize(ctx->prof_mark[i]));
    float ms = 0.f;
    VLAC_HIP(hipEventElapsedTime(&ms, ctx->prof_start[i], ctx->prof_stop[i]));
    tot += ms;
    VLAC_HIP(hipEventElapsedTime(&ms, ctx->prof_stop[i], ctx->prof_mark[i]));
    mark += ms;
  }
  *total_ms = tot;
  if (marker_ms) *marker_ms = mark;
  *launches = ctx->prof_n;
  ctx->prof_n = 0;
  return VLAC_OK;
}

int vlac_profile_read(vlac_ctx* ctx, double* total_ms, int* launches) {
  return vlac_profile_read2(ctx, total_ms, nullptr, launches);
}

int vlac_profile_bracket_cost(vlac_ctx* ctx, void* stream, double* cost_us) {
  if (!ctx || !cost_us) return VLAC_E_NULL;
  constexpr int N = 40, SKIP = 8;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t ev[2 * N];
  int made = 0, rc = VLAC_OK;
  unsigned long long self[N];
  unsigned long long* d_self = (unsigned long long*)ctx->partial;  // idle between launches
  for (; made < 2 * N; ++made)
    if (hipEventCreate(&ev[made]) != hipSuccess) { rc = VLAC_E_HIP; break; }
  if (rc == VLAC_OK) {
    for (int i = 0; i < N; ++i) {
      (void)hipEventRecord(ev[2 * i], st);
      hipLaunchKernelGGL(spin_kernel, dim3(1), dim3(64), 0, st, 2000ull, d_self + i);  // 20 us
      (void)hipEventRecord(ev[2 * i + 1], st);
    }
    if (hipMemcpyAsync(self, d_self, sizeof(self), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) rc = VLAC_E_HIP;
  }
  if (rc == VLAC_OK) {
    double sum = 0;
    for (int i = SKIP; i < N; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) { rc = VLAC_E_HIP; break; }
      sum += (double)ms * 1e3 - (double)self[i] * 0.01;  // the wall clock counts at 100 MHz
    }
    *cost_us = sum / (N - SKIP);
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
  return rc;
}

int vlac_check(vlac_ctx* ctx, void* stream) {
  if (!ctx) return VLAC_E_NULL;
  int word = 0;
  VLAC_HIP(hipMemcpyAsync(&word, ctx->errword, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream));
  VLAC_HIP(hipStreamSynchronize((hipStream_t)stream));
  if (word) {
    VLAC_HIP(hipMemsetAsync(ctx->errword, 0, sizeof(int), (hipStream_t)stream));
    VLAC_HIP(hipStreamSynchronize((hipStream_t)stream));
    return VLAC_E_RANGE;
  }
  return VLAC_OK;
}

int vlac_embed_patches(vlac_ctx* ctx, const uint8_t* frame_cur, int B, int H, int W, int patch,
                       const void* w_proj, const int32_t* reuse_order, const int32_t* reuse_count,
                       int stride, const int32_t* layer_count, float* embeds, int L, void* stream) {
  if (!ctx || !frame_cur || !w_proj || !embeds) return VLAC_E_NULL;
  if ((reuse_order == nullptr) != (reuse_count == nullptr)) return VLAC_E_NULL;
  if (layer_count && !reuse_order) return VLAC_E_NULL;
  if (B < 1 || B > ctx->cfg.max_batch) return VLAC_E_RANGE;
  // (8 patches of fp32 pixels are staged in 64 KiB of LDS: 3 patch^2 <= 2048)
  if (patch < 1 || patch > 26 || H < patch || W < patch || H % patch || W % patch) return VLAC_E_SHAPE;
  const long long L_v = (long long)(H / patch) * (W / patch);
  if (L_v > 4096 || L < L_v) return VLAC_E_SHAPE;
  if (reuse_order && stride < 1) return VLAC_E_RANGE;
  launch_embed_patches(ctx, frame_cur, B, H, W, patch, (const bf16_t*)w_proj, reuse_order, reuse_count,
                       stride, layer_count, embeds, L, (hipStream_t)stream);
  VLAC_HIP(hipGetLastError());
  return VLAC_OK;
}

int vlac_select_static(vlac_ctx* ctx, const uint8_t* frame_prev, const uint8_t* frame_cur, int B,
                       int H, int W, int patch, int tau_num, int tau_den, int top_k,
                       const float* attn_mean, const uint8_t* layer_mask, float tau_task,
                       int32_t* out_idx, int32_t* out_order, int32_t* out_count,
                       float* out_relevance, int stride, void* stream) {
  if (!ctx || !frame_prev || !frame_cur || !out_idx || !out_order || !out_count) return VLAC_E_NULL;
  if (B < 1 || B > ctx->cfg.max_batch) return VLAC_E_RANGE;
  if (patch < 1 || patch > 64 || H < 1 || W < 1) return VLAC_E_RANGE;
  if (H % patch || W % patch) return VLAC_E_SHAPE;
  const long L_v = (long)(H / patch) * (W / patch);
  if (L_v > 4096) return VLAC_E_RANGE;
  if (tau_den < 1 || tau_num < 0 || tau_num > tau_den) return VLAC_E_RANGE;
  if (top_k < 0 || top_k > L_v) return VLAC_E_RANGE;
  if (stride < top_k || stride < 1) return VLAC_E_SHAPE;
  if (tau_task != tau_task) return VLAC_E_RANGE;  // NaN
  int n_rel = 0;
  if (attn_mean) {
    // the L_v - floor(tau_task * L_v) highest-scoring tokens are task-relevant
    const double keep = floor((double)tau_task * (double)L_v);
    double nr = (double)L_v - keep;
    n_rel = nr < 0 ? 0 : (nr > (double)L_v ? (int)L_v : (int)nr);
  }
  hipStream_t st = (hipStream_t)stream;
  launch_patch_terms(frame_prev, frame_cur, B, H, W, patch, ctx->terms, st);
  launch_select(ctx->terms, B, (int)L_v, tau_num, tau_den, top_k, attn_mean, ctx->cfg.n_layers,
                layer_mask, n_rel, ctx->flags, ctx->relevance, out_idx, out_order, out_count,
                out_relevance, stride, st);
  VLAC_HIP(hipGetLastError());
  return VLAC_OK;
}

int vlac_layer_ratio(vlac_ctx* ctx, const float* attn_mean, int B, int L_v, float gain_k,
                     const int32_t* reuse_count, float* out_alpha, int32_t* out_layer_count,
                     void* stream) {
  if (!ctx || !attn_mean || !out_alpha) return VLAC_E_NULL;
  if (out_layer_count && !reuse_count) return VLAC_E_NULL;
  if (B < 1 || B > ctx->cfg.max_batch || L_v < 1 || L_v > 65536) return VLAC_E_RANGE;
  if (gain_k != gain_k) return VLAC_E_RANGE;
  launch_layer_ratio(attn_mean, ctx->cfg.n_layers, B, L_v, gain_k, reuse_count, out_alpha,
                     out_layer_count, (hipStream_t)stream);
  VLAC_HIP(hipGetLastError());
  return VLAC_OK;
}

}  // extern "C"

namespace {

// One decoder layer over the rows of plane `rows` (count *n_rows <= rows_cap).
// n_host >= 0: the row count is known on the host; decode_pos >= 0: the rows are
// (stream b, position decode_pos) for b < n_host, and the row lists are not read.
// *pending: split-K factor of partial rows (in c->rpart) that still have to be added
// to the residual stream c->h: on entry from the previous layer's FFN, on exit from
// this layer's FFN (0: the residual stream is complete).
void run_layer(vlac_ctx* c, int layer, int B, int rows_cap, int rows_cap_per_stream, int L_v, int L_t,
               const float* resid_in, int resid_stride, const int* rows, const int* n_rows,
               int n_host, int decode_pos, const int* slot_off, const int* prev_slot, bf16_t* kv,
               float* out_attn_mean, int* pending, hipStream_t st) {
  const vlac_model_cfg& m = c->cfg;
  const LayerW& W = c->layers[layer];
  GemmEpi e;
  memset(&e, 0, sizeof(e));
  e.rows = rows;
  e.decode_pos = decode_pos;
  e.rope_cos = c->rope_cos; e.rope_sin = c->rope_sin;
  e.qbuf = c->qbuf;
  e.kv = kv;
  e.kv_stream_stride = kv_elems_per_stream(m);
  e.kv_layer_off = (size_t)layer * 2 * m.n_kv_heads * m.max_seq * m.head_dim;
  e.n_q_heads = m.n_q_heads; e.n_kv_heads = m.n_kv_heads; e.head_dim = m.head_dim;
  e.max_seq = m.max_seq;
  e.h = c->h; e.h_seq_stride = m.max_seq; e.d_model = m.d_model;
  e.rpart = c->rpart; e.rpart_rows = rows_cap;
  e.xf = c->xf; e.kc_f = c->kpad_f / 16; e.d_ffn = m.d_ffn;
  const int kc_d = c->kpad_d / 16;

  if (*pending)
    launch_resid_norm_rows(c->f16, c->h, m.max_seq, c->rpart, *pending, rows_cap, c->h, m.max_seq,
                           rows, prev_slot, n_rows, n_host, rows_cap, W.g_attn, m.rms_eps,
                           m.d_model, c->xa, kc_d, st, &c->pending_adapt);
  else
    launch_rmsnorm_rows(c->f16, resid_in, resid_stride, rows, n_rows, n_host, decode_pos, rows_cap,
                        W.g_attn, m.rms_eps, m.d_model, c->xa, kc_d, st);
  launch_gemm(c, EPI_QKV, W.wqkv, W.s_qkv, c->qkv_dim / 32, c->kpad_d, c->xa, n_rows, n_host, rows_cap, e, st);
  *pending = 0;
  launch_attention(c, layer, B, rows_cap_per_stream, L_v, L_t, rows, slot_off, decode_pos, kv,
                   out_attn_mean, st);
  e.resid_src = resid_in; e.resid_seq_stride = resid_stride;
  const int s_o = launch_gemm(c, EPI_RESID, W.wo, W.s_o, m.d_model / 32, c->kpad_q, c->xa, n_rows, n_host,
                              rows_cap, e, st);
  const SplitAdapt ad_o = gemm_resid_adapt(c, m.d_model / 32, c->kpad_q, rows_cap, n_rows, n_host);
  if (rows_cap > 32 && s_o > 1)  // the few-rows kernel adds its splits up itself
    launch_resid_norm_rows(c->f16, resid_in, resid_stride, c->rpart, s_o, rows_cap, c->h, m.max_seq,
                           rows, nullptr, n_rows, n_host, rows_cap, W.g_ffn, m.rms_eps, m.d_model,
                           c->xa, kc_d, st, &ad_o);
  else
    launch_rmsnorm_rows(c->f16, c->h, m.max_seq, rows, n_rows, n_host, decode_pos, rows_cap, W.g_ffn,
                        m.rms_eps, m.d_model, c->xa, kc_d, st);
  launch_gemm(c, EPI_SWIGLU, W.wgu, W.s_gu, 2 * m.d_ffn / 32, c->kpad_d, c->xa, n_rows, n_host, rows_cap, e, st);
  e.resid_src = c->h; e.resid_seq_stride = m.max_seq;
  const int s_d = launch_gemm(c, EPI_RESID, W.wdown, W.s_down, m.d_model / 32, c->kpad_f, c->xf, n_rows, n_host,
                              rows_cap, e, st);
  *pending = (rows_cap > 32 && s_d > 1) ? s_d : 0;
  c->pending_adapt = gemm_resid_adapt(c, m.d_model / 32, c->kpad_f, rows_cap, n_rows, n_host);
}

// The residual rows of a decode pass with at most 4 streams: one row per stream in one
// of the two row sets of c->hdec.  `pending` > 0: the rows are not complete yet, that
// many split-K partial rows per stream (in c->rpart) have to be added first, which the
// next fused norm does, storing the completed rows in the other set.
struct DecodeResid {
  int cur, pending;
};

NormIn decode_norm(vlac_ctx* c, int B, DecodeResid& r, const float* gain, bool keep) {
  const int d = c->cfg.d_model;
  NormIn n;
  memset(&n, 0, sizeof(n));
  n.src = c->hdec + (size_t)r.cur * c->cfg.max_batch * d;
  n.src_stride = d;
  n.gain = gain;
  n.eps = c->cfg.rms_eps;
  n.d = d;
  if (r.pending) {
    n.part = c->rpart; n.part_S = r.pending; n.part_rows = B;
    if (keep) {
      r.cur ^= 1;
      n.dst = c->hdec + (size_t)r.cur * c->cfg.max_batch * d;
      n.dst_stride = d;
    }
    r.pending = 0;
  }
  return n;
}

// One decoder layer of a decode pass over the rows (stream b, position pos), b < B <= 4:
// every RMSNorm is fused into the GEMM that follows it, and the two projections with a
// residual leave their split-K partial rows to the next norm (no hand-over inside them).
void run_layer_decode(vlac_ctx* c, int layer, int B, int pos, bf16_t* kv, DecodeResid& r,
                      hipStream_t st) {
  const vlac_model_cfg& m = c->cfg;
  const LayerW& W = c->layers[layer];
  GemmEpi e;
  memset(&e, 0, sizeof(e));
  e.decode_pos = pos;
  e.rope_cos = c->rope_cos; e.rope_sin = c->rope_sin;
  e.qbuf = c->qbuf;
  e.kv = kv;
  e.kv_stream_stride = kv_elems_per_stream(m);
  e.kv_layer_off = (size_t)layer * 2 * m.n_kv_heads * m.max_seq * m.head_dim;
  e.n_q_heads = m.n_q_heads; e.n_kv_heads = m.n_kv_heads; e.head_dim = m.head_dim;
  e.max_seq = m.max_seq;
  e.d_model = m.d_model;
  e.h_compact = 1; e.h_seq_stride = 1; e.resid_seq_stride = 1;
  e.rpart = c->rpart; e.rpart_rows = B; e.defer_split = 1;
  e.xf = c->xf; e.kc_f = c->kpad_f / 16; e.d_ffn = m.d_ffn;

  NormIn n = decode_norm(c, B, r, W.g_attn, true);
  launch_gemm(c, EPI_QKV, W.wqkv, W.s_qkv, c->qkv_dim / 32, c->kpad_d, c->xa, nullptr, B, B, e, st, &n);
  launch_attention(c, layer, B, 1, 0, 0, nullptr, nullptr, pos, kv, nullptr, st);
  float* hrow = c->hdec + (size_t)r.cur * m.max_batch * m.d_model;
  e.resid_src = hrow; e.h = hrow;
  const int s_o = launch_gemm(c, EPI_RESID, W.wo, W.s_o, m.d_model / 32, c->kpad_q, c->xa, nullptr, B, B, e, st);
  r.pending = s_o > 1 ? s_o : 0;
  n = decode_norm(c, B, r, W.g_ffn, true);
  launch_gemm(c, EPI_SWIGLU, W.wgu, W.s_gu, 2 * m.d_ffn / 32, c->kpad_d, c->xa, nullptr, B, B, e, st, &n);
  hrow = c->hdec + (size_t)r.cur * m.max_batch * m.d_model;
  e.resid_src = hrow; e.h = hrow;
  const int s_d = launch_gemm(c, EPI_RESID, W.wdown, W.s_down, m.d_model / 32, c->kpad_f, c->xf, nullptr, B, B, e, st);
  r.pending = s_d > 1 ? s_d : 0;
}

// Final norm + output head + greedy token for B rows: (stream b, position pos) of the
// residual stream, or, with `fused` given, the rows of a decode pass (norm fused).
void run_head(vlac_ctx* c, int B, int pos, float* logits, size_t logits_stride, int32_t* out_token,
              int out_stride, int32_t* token_copy, hipStream_t st, const NormIn* fused = nullptr) {
  const vlac_model_cfg& m = c->cfg;
  GemmEpi e;
  memset(&e, 0, sizeof(e));
  e.decode_pos = pos;
  e.logits = logits; e.vocab = m.vocab; e.logits_stride = logits_stride;
  if (fused) {
    launch_gemm(c, EPI_LOGITS, c->w_head, c->s_head, m.vocab / 32, c->kpad_d, c->xa, nullptr, B, B, e, st, fused);
  } else if (gemm_can_fuse_norm(B, pos, c->kpad_d)) {
    NormIn n;
    memset(&n, 0, sizeof(n));
    n.src = c->h + (size_t)pos * m.d_model; n.src_stride = (size_t)m.max_seq * m.d_model;
    n.gain = c->g_final; n.eps = m.rms_eps; n.d = m.d_model;
    launch_gemm(c, EPI_LOGITS, c->w_head, c->s_head, m.vocab / 32, c->kpad_d, c->xa, nullptr, B, B, e, st, &n);
  } else {
    launch_rmsnorm_rows(c->f16, c->h, m.max_seq, nullptr, nullptr, B, pos, B, c->g_final, m.rms_eps,
                        m.d_model, c->xa, c->kpad_d / 16, st);
    launch_gemm(c, EPI_LOGITS, c->w_head, c->s_head, m.vocab / 32, c->kpad_d, c->xa, nullptr, B, B, e, st);
  }
  launch_argmax(logits, logits_stride, B, m.vocab, out_token, out_stride, token_copy, st);
}

int weights_ready(const vlac_ctx* c) {
  if (!c->head_set) return 0;
  for (int l = 0; l < c->cfg.n_layers; ++l)
    if (!c->layer_set[l]) return 0;
  return 1;
}

}  // namespace

extern "C" {

int vlac_sparse_prefill(vlac_ctx* ctx, const float* embeds, int B, int L_v, int L_t,
                        const int32_t* reuse_order, const int32_t* reuse_count, int stride,
                        const int32_t* layer_count, void* kv_cache, float* out_attn_mean,
                        float* out_hidden, float* out_logits, int32_t* out_token, void* stream) {
  if (!ctx || !embeds || !kv_cache || !out_token) return VLAC_E_NULL;
  if ((reuse_order == nullptr) != (reuse_count == nullptr)) return VLAC_E_NULL;
  if (layer_count && !reuse_count) return VLAC_E_NULL;
  const vlac_model_cfg& m = ctx->cfg;
  if (B < 1 || B > m.max_batch) return VLAC_E_RANGE;
  if (L_v < 0 || L_t < 0 || L_v + L_t < 1) return VLAC_E_RANGE;
  const int L = L_v + L_t;
  if (L > m.max_seq) return VLAC_E_SHAPE;
  if (reuse_order && (stride < 1 || L_v < 1)) return VLAC_E_SHAPE;
  if (!weights_ready(ctx)) return VLAC_E_STATE;
  for (int b = 0; b < B; ++b) {
    if (!ctx->was_reset[b]) return VLAC_E_STATE;
    if (reuse_order && !ctx->filled[b]) return VLAC_E_STATE;
  }
  hipStream_t st = (hipStream_t)stream;
  const int nl = m.n_layers;
  launch_plan(ctx, B, L_v, L_t, reuse_order, reuse_count, stride, layer_count, st);
  const int rows_cap = B * L;
  const int n_host = reuse_order ? -1 : rows_cap;
  // (a stream reuses at most `stride` tokens: its list has no room for more)
  ctx->rows_floor = reuse_order ? B * (L - (stride < L_v ? stride : L_v)) : rows_cap;
  int pending = 0;
  for (int l = 0; l < nl; ++l) {
    const int* rows = ctx->rows + (size_t)l * ctx->max_rows;
    run_layer(ctx, l, B, rows_cap, L, L_v, L_t, l == 0 ? embeds : ctx->h, l == 0 ? L : m.max_seq,
              rows, ctx->n_rows + l, n_host, -1, ctx->slot_off + (size_t)l * (m.max_batch + 1),
              ctx->prev_slot + (size_t)l * ctx->max_rows, (bf16_t*)kv_cache, out_attn_mean, &pending,
              st);
  }
  if (pending)  // the last FFN's partial rows still have to reach the residual stream
    launch_resid_norm_rows(ctx->f16, ctx->h, m.max_seq, ctx->rpart, pending, rows_cap, ctx->h,
                           m.max_seq, ctx->rows + (size_t)(nl - 1) * ctx->max_rows, nullptr,
                           ctx->n_rows + (nl - 1), n_host, rows_cap, nullptr, m.rms_eps, m.d_model,
                           ctx->xa, ctx->kpad_d / 16, st, &ctx->pending_adapt);
  if (out_attn_mean && attention_defers_stats(ctx, B, L_v, L_t))
    launch_stats_reduce(ctx, B, L_v, L_t, out_attn_mean, st);
  if (out_hidden)
    launch_final_hidden(ctx->h, m.max_seq, ctx->rows + (size_t)(nl - 1) * ctx->max_rows,
                        ctx->n_rows + (nl - 1), rows_cap, ctx->g_final, m.rms_eps, m.d_model,
                        out_hidden, L, st);
  run_head(ctx, B, L - 1, out_logits ? out_logits : ctx->logits, (size_t)m.vocab, out_token, 1,
           nullptr, st);
  VLAC_HIP(hipGetLastError());
  for (int b = 0; b < B; ++b) ctx->filled[b] = 1;
  return VLAC_OK;
}

int vlac_decode_action(vlac_ctx* ctx, int B, int L, int n_new, const int32_t* first_token,
                       void* kv_cache, int32_t* out_tokens, float* out_logits, void* stream) {
  if (!ctx || !first_token || !kv_cache || !out_tokens) return VLAC_E_NULL;
  const vlac_model_cfg& m = ctx->cfg;
  if (B < 1 || B > m.max_batch || L < 1 || n_new < 0) return VLAC_E_RANGE;
  if ((long)L + n_new > m.max_seq) return VLAC_E_SHAPE;
  if (!weights_ready(ctx)) return VLAC_E_STATE;
  for (int b = 0; b < B; ++b)
    if (!ctx->filled[b]) return VLAC_E_STATE;
  if (n_new == 0) return VLAC_OK;
  hipStream_t st = (hipStream_t)stream;
  const int ms = m.max_seq;
  const bool fused = gemm_can_fuse_norm(B, L, ctx->kpad_d) && ctx->rpart_floats >= (size_t)8 * B * m.d_model;
  if (!fused) launch_decode_plan(ctx, B, L, n_new, st);
  for (int t = 0; t < n_new; ++t) {
    const int32_t* tok = t == 0 ? first_token : ctx->tokens;
    float* logits = out_logits ? out_logits + (size_t)t * m.vocab : ctx->logits;
    const size_t lstride = out_logits ? (size_t)n_new * m.vocab : (size_t)m.vocab;
    if (fused) {
      // rows (b, 0) of a [max_batch, 1, d] plane: the first residual row set
      launch_embed_rows(ctx->embed, tok, B, m.d_model, m.vocab, ctx->hdec, 1, 0, st);
      DecodeResid r = {0, 0};
      for (int l = 0; l < m.n_layers; ++l)
        run_layer_decode(ctx, l, B, L + t, (bf16_t*)kv_cache, r, st);
      const NormIn n = decode_norm(ctx, B, r, ctx->g_final, false);
      run_head(ctx, B, L + t, logits, lstride, out_tokens + t, n_new, ctx->tokens, st, &n);
    } else {
      // More than 4 streams: the general layer pass over the rows (b, L + t).  With more than
      // 32 of them the prefill's GEMM and row kernels serve the pass, and those read the row
      // list (only the few-rows kernels derive a row from decode_pos): plane t of the decode
      // row lists.  Their projections with a residual may leave split-K partial rows
      // (`pending`), which the next layer's first row kernel adds up, and after the last
      // layer a row kernel without a norm.
      launch_embed_rows(ctx->embed, tok, B, m.d_model, m.vocab, ctx->h, ms, L + t, st);
      const int* drows = ctx->dec_rows + (size_t)t * m.max_batch;
      int pending = 0;
      for (int l = 0; l < m.n_layers; ++l)
        run_layer(ctx, l, B, B, 1, 0, 0, ctx->h, ms, drows, nullptr, B, L + t, nullptr, nullptr,
                  (bf16_t*)kv_cache, nullptr, &pending, st);
      if (pending)
        launch_resid_norm_rows(ctx->f16, ctx->h, ms, ctx->rpart, pending, B, ctx->h, ms, drows, nullptr,
                               nullptr, B, B, nullptr, m.rms_eps, m.d_model, ctx->xa, ctx->kpad_d / 16,
                               st, &ctx->pending_adapt);
      run_head(ctx, B, L + t, logits, lstride, out_tokens + t, n_new, ctx->tokens, st);
    }
  }
  VLAC_HIP(hipGetLastError());
  return VLAC_OK;
}

}  // extern "C"
