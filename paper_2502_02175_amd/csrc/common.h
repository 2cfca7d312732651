// Internal declarations shared by the kernels and the C-ABI layer of vlac.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vlac.h"

typedef uint16_t bf16_t;  // raw bf16 bits

// ---------------------------------------------------------------------------
// Fragment order.  Every bf16 operand of a matrix-core GEMM ([R rows, K cols],
// weights and activations alike) is stored as tiles of 32 rows x 16 cols.  A
// tile is 1 KiB: 64 lanes x 8 bf16, lane = (row % 32) + 32 * ((col % 16) / 8),
// element = col % 8, which is exactly what one v_mfma_f32_32x32x16_bf16 operand
// wants per lane, so a wave fetches a tile with one coalesced 16-byte load per
// lane.  Tiles are ordered [row tile][col tile]; KC = padded K / 16.
// ---------------------------------------------------------------------------
__host__ __device__ inline size_t frag_off(int row, int col, int KC) {
  return ((size_t)(row >> 5) * KC + (col >> 4)) * 512 +
         (size_t)((((row & 31) + (((col >> 3) & 1) << 5)) << 3) + (col & 7));
}

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

#ifdef __HIPCC__
// Matrix-core operands are 16-bit: bf16 (F16 = false) or IEEE fp16 (F16 = true).
// The weights arrive as bf16; every bf16 value of ordinary magnitude is exactly
// representable in fp16 (7 mantissa bits fit in 10), so the fp16 mode only
// changes how finely the ACTIVATIONS are rounded (2^-11 instead of 2^-8 relative).
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ inline bf16_t f2bf(float x) {  // fp32 -> bf16, round to nearest even
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ inline uint16_t f2h(float x) {  // fp32 -> fp16, round to nearest even, saturating
  const _Float16 h = (_Float16)fminf(fmaxf(x, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, h);
}
template <bool F16>
__device__ inline uint16_t f2op(float x) {
  if constexpr (F16) return f2h(x);
  else return f2bf(x);
}
template <bool F16>
__device__ inline uint32_t pack_op2(float lo, float hi) {
  return (uint32_t)f2op<F16>(lo) | ((uint32_t)f2op<F16>(hi) << 16);
}
// Hand-over of partial results between workgroups (split-K sums, attention
// statistics).  The 8 XCDs have one L2 each, and an agent-scope fence
// (__threadfence) writes back and invalidates a whole L2, which costs more than
// the kernels it would sit in.  Instead the few words that change hands are
// written and read with agent-scope atomic accesses, which go through to the
// memory side and bypass stale lines.  Before the arrival counter is bumped, every wave
// waits until its stores have been acknowledged (s_waitcnt vmcnt(0), stores count there
// on this chip): the workgroup-scope fence that follows does NOT wait for them by itself
// (the waves of a workgroup share their L1, so the compiler omits the wait), and without
// it the counter can overtake a store on its way to another L2 channel: the last
// workgroup to arrive then reads what the location held before (seen about once in 400
// prefills of 224 launches each).
__device__ inline void st_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void stores_done() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
}

// D[32x32] += A[32x16] . B[16x32]; a lane supplies 8 consecutive k of row/col (lane % 32)
template <bool F16>
__device__ inline f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
#endif

// Hand-placed waits for copies that the compiler does not see (global -> LDS copies written
// as inline assembly): "at most n vector-memory operations outstanding".  A build with
// -DVLAC_SAFE_WAITS waits for all of them instead; it computes the same values in the same
// order, so its results must equal the normal build's bit for bit, and a miscounted wait (an
// LDS read before its tile has landed) shows as a difference between the two builds.
#ifdef VLAC_SAFE_WAITS
#define VLAC_VMCNT(n) asm volatile("s_waitcnt vmcnt(0)" ::: "memory")
#else
#define VLAC_VMCNT(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")
#endif

enum { VLAC_ERR_BAD_INDEX = 1 };  // bits of the device-side error word

struct LayerW {
  bf16_t *wqkv, *wo, *wgu, *wdown;  // fragment order (16-bit operands, or e4m3 codes)
  float *g_attn, *g_ffn;
  float *s_qkv, *s_o, *s_gu, *s_down;  // e4m3 weights: scale per packed output row
};

// What launch_resid_norm_rows needs to know of the GEMM whose partial rows it adds up, where
// that GEMM chooses its split factor on the device (n_blocks == 0: the factor is S as given)
struct SplitAdapt {
  const int* n_rows;  // device: the row count the GEMM ran with (n_rows_host >= 0: not read)
  int n_rows_host, n_blocks, KS;  // the GEMM's feature blocks and 64-k steps
  int S_tall;         // most splits the many-rows kernel may have used (tall_plan)
  int small_below;    // > 0: with fewer rows than this the one-stream kernel ran instead ...
  int S_small;        // ... and split K in this many parts (1: it completed the rows itself)
};

struct vlac_ctx {
  vlac_model_cfg cfg;
  bool f16;  // operands are fp16 (else bf16)
  bool w8;   // weights are stored as e4m3 codes + a scale per output feature (f16 operands)
  int device;
  int last_hip;
  // derived
  int q_dim, kv_dim, qkv_dim, group;
  int kpad_d, kpad_q, kpad_f;  // K padded to 64 for d_model, Hq*hd, d_ffn
  int max_rows;                // max_batch * max_seq
  // weights
  LayerW* layers;  // host array
  uint8_t* layer_set;
  bool head_set;
  bf16_t *w_head, *embed;
  float* s_head;
  float* scale_tmp;  // scales in source row order while a matrix is being packed
  bf16_t* wdeq;      // e4m3 weights, many rows: one matrix expanded to fp16 for the many-rows GEMM
  int rows_floor;    // fewest rows the prefill that is being launched can have (from the reuse lists' length)
  SplitAdapt pending_adapt;  // of the FFN-down GEMM whose partial rows the next layer's first row kernel adds
  float* g_final;
  float *rope_cos, *rope_sin;  // [max_seq, hd/2]
  // workspace (device)
  float* h;         // residual stream [max_batch, max_seq, d]
  float* hdec;      // decode with the fused norm: two residual row sets [2][max_batch, d]
  bf16_t* xa;       // normed rows / attention output, fragment order
  bf16_t* xf;       // SwiGLU output, fragment order
  bf16_t* qbuf;     // rotated queries, fragment order per head
  float* partial;   // split-K partial sums
  size_t partial_floats;
  float* rpart;     // split-K partial rows of the projection + residual GEMMs
  size_t rpart_floats;
  int* counters;    // split-K arrival counters (self-resetting)
  int n_counters;
  int* rows;        // [n_layers + 1][max_rows] (b << 16 | pos); last plane: head rows
  int* prev_slot;   // [n_layers][max_rows] slot of the same row in the previous layer's list
  int* n_rows;      // [n_layers + 1]
  int* slot_off;    // [n_layers + 1][max_batch + 1]
  int* rank;        // [max_batch][max_seq] position of a token in its reuse order
  int* m_layer;     // [max_batch][n_layers]
  int* n_rows_bl;   // [n_layers][max_batch]
  float* statp;     // attention-statistic partial sums
  size_t statp_floats;
  int stat_tt;      // text tiles per stream the statistic buffer provides for
  int* stat_counters;
  float* logits;    // [max_batch, vocab]
  int* tokens;      // [max_batch] current token of the decode loop
  int* dec_rows;    // decode row lists
  uint32_t* terms;  // patch terms [max_batch, 4096, 3]
  uint8_t* flags;   // selection flags
  int* embed_list;  // [max_batch][4096] patches to embed
  int* embed_n;     // [max_batch]
  float* relevance; // [max_batch, 4096]
  bf16_t* zero_tile; // one operand tile of zeros
  int* errword;     // device error bits
  int* scratch_i;   // small int scratch
  uint8_t* filled;  // host: stream cache holds a prefill
  uint8_t* was_reset;
  // per-launch timing of one GEMM class (vlac_profile_select)
  int prof_kind, prof_n, prof_cap;
  hipEvent_t *prof_start, *prof_stop, *prof_mark;
};

#define VLAC_HIP(call)                         \
  do {                                         \
    hipError_t e_ = (call);                    \
    if (e_ != hipSuccess) {                    \
      if (ctx) ctx->last_hip = (int)e_;        \
      return VLAC_E_HIP;                       \
    }                                          \
  } while (0)

// ---- launchers implemented in the .hip files (all asynchronous on `st`) ----

// select.hip
void launch_patch_terms(const uint8_t* prev, const uint8_t* cur, int B, int H, int W, int patch,
                        uint32_t* terms, hipStream_t st);
void launch_select(const uint32_t* terms, int B, int L_v, int tau_num, int tau_den, int top_k,
                   const float* attn_mean, int n_layers, const uint8_t* layer_mask_host, int n_rel,
                   uint8_t* flags, float* relevance_ws, int32_t* out_idx, int32_t* out_order,
                   int32_t* out_count, float* out_relevance, int stride, hipStream_t st);
int select_scratch_init();  // resolves the fixed scratch of vlac_select_static_noalloc on the current device; hipError_t
void launch_layer_ratio(const float* attn_mean, int n_layers, int B, int L_v, float gain_k,
                        const int32_t* reuse_count, float* out_alpha, int32_t* out_layer_count,
                        hipStream_t st);

// rows.hip
void launch_plan(vlac_ctx* c, int B, int L_v, int L_t, const int32_t* reuse_order,
                 const int32_t* reuse_count, int stride, const int32_t* layer_count, hipStream_t st);
void launch_decode_plan(vlac_ctx* c, int B, int L, int n_new, hipStream_t st);
void launch_rmsnorm_rows(bool f16, const float* src, int seq_stride, const int* rows,
                         const int* n_rows, int n_rows_host, int decode_pos, int max_rows, const float* gain, float eps, int d,
                         bf16_t* xp, int KC, hipStream_t st);
// h[row] = resid[row] + sum of the S partial rows; optionally RMSNorm(h[row]) -> operand xp
void launch_resid_norm_rows(bool f16, const float* resid, int resid_seq_stride, const float* part,
                            int S, int part_rows, float* h, int h_seq_stride, const int* rows,
                            const int* part_slot, const int* n_rows, int n_rows_host, int max_rows,
                            const float* gain, float eps, int d, bf16_t* xp, int KC,
                            hipStream_t st, const SplitAdapt* adapt = nullptr);
void launch_final_hidden(const float* src, int seq_stride, const int* rows, const int* n_rows,
                         int max_rows, const float* gain, float eps, int d, float* out, int L,
                         hipStream_t st);
void launch_argmax(const float* logits, size_t logits_stride, int B, int vocab, int32_t* out,
                   int out_stride, int32_t* out2, hipStream_t st);
void launch_embed_rows(const bf16_t* embed, const int32_t* tokens, int B, int d, int vocab, float* h,
                       int max_seq, int pos, hipStream_t st);
// e4m3 storage: scales of the N source rows, then codes in fragment order (two k-tiles per
// 16-byte lane slot) and the scales in packed row order
void launch_row_scales(const bf16_t* src, int N, int K, float* scales, hipStream_t st);
void launch_pack_e4m3(const bf16_t* src, int N, int K, const float* scales, bf16_t* dst, float* scales_packed,
                      int n_pack, int kpad, int mode, int p0, int p1, int p2, hipStream_t st);
void launch_quantize_e4m3(const bf16_t* src, int N, int K, const float* scales, uint8_t* codes, hipStream_t st);
void launch_pack(bool to_f16, const bf16_t* src, int N, int K, bf16_t* dst, int n_pack, int kpad,
                 int mode, int p0, int p1, int p2, hipStream_t st);
void launch_bf16_to_f32(const bf16_t* src, float* dst, int n, hipStream_t st);

// gemm.hip
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };
struct GemmEpi {
  const int* rows;
  int decode_pos;  // >= 0: row `slot` is (stream slot, position decode_pos), rows is not read
  // EPI_QKV
  const float *rope_cos, *rope_sin;
  bf16_t* qbuf;
  bf16_t* kv;             // cache base of layer 0, stream 0
  size_t kv_stream_stride, kv_layer_off;
  int n_q_heads, n_kv_heads, head_dim, max_seq;
  // EPI_RESID: h[b][pos] = resid_src[b][pos] + projection; rows of h_seq_stride /
  // resid_seq_stride positions per stream (h_compact: one row per stream, pos is ignored)
  const float* resid_src; int resid_seq_stride;
  float* h; int h_seq_stride; int h_compact; int d_model;
  float* rpart; int rpart_rows;  // split-K partial rows [split][rpart_rows][d_model]
  int defer_split;  // few-rows kernel with S > 1: leave the partial rows in rpart
  // EPI_SWIGLU
  bf16_t* xf; int kc_f; int d_ffn;
  // EPI_LOGITS
  float* logits; int vocab; size_t logits_stride;  // elements between rows
};
// RMSNorm fused into the few-rows GEMM: x = src row (+ split-K partial rows, in split
// order), operand = x * rsqrt(mean(x^2) + eps) * gain
struct NormIn {
  const float* src;    // row 0 of the fp32 source rows
  size_t src_stride;   // floats between consecutive rows
  const float* gain;
  float eps;
  int d;
  const float* part;   // partial rows [part_S][part_rows][d] still to be added, or null
  int part_S, part_rows;
  float* dst;          // where the completed rows are stored (never src), or null
  size_t dst_stride;
};
// The many-rows kernel with both operands through LDS (gemm_tall.hip) cuts the rows of a
// launch into blocks of 256, 192 or 128 rows (a work item is 256 features wide and fetches 16,
// 14 or 12 KiB of operands per k-tile for 64, 48 or 32 MFMAs) and, where the projection adds
// to the residual stream, K into up to S_max parts whose partial rows the row kernel that
// follows adds up; the cut follows from the ACTUAL row count, on the device.  Taken is the cut
// with the least estimated time: rounds of 256 work items x the KiB an item moves (its
// operands over its share of K; with K split also its partial rows, written once and read once
// by the row kernel: 2 x 64 rt rows x 256 features x 4 bytes, counted twice, because they go
// through memory where operand tiles are mostly shared in L2); ties go to the larger block
// and the fewer parts.  KS: 64-k steps of the projection.  Both the GEMM and the row kernel
// that consumes the partial rows call this function (32-bit arithmetic, divisions by
// constants only).
struct TallPlan {
  int rt, tiles, row_blocks, S;  // row tiles per wave (4, 3 or 2), weight tiles of 256 features, row blocks, K parts
  __host__ __device__ int items() const { return tiles * S * row_blocks; }
};
__host__ __device__ inline TallPlan tall_plan(int tiles, int n_rows, int S_max, int KS) {
  TallPlan p;
  p.tiles = tiles;
  p.rt = 4;
  p.S = 1;
  p.row_blocks = (n_rows + 255) >> 8;
  if (S_max > 8) S_max = 8;
  if (S_max < 1 || KS < 24) S_max = 1;
  if (KS > 8192) KS = 8192;  // (keeps the estimate inside 32 bits; the choice no longer depends on K there)
  unsigned best = 0xffffffffu;
#define VLAC_TALL_TRY(S_, RT_)                                                                     \
  if (S_ <= S_max) {                                                                             \
    const unsigned rb = ((unsigned)n_rows + 64u * RT_ - 1u) / (64u * RT_);                       \
    unsigned rounds = ((unsigned)tiles * S_ * rb + 255u) >> 8;                                   \
    if (rounds > 4096u) rounds = 4096u;                                                          \
    const unsigned steps = (2u * (unsigned)KS + S_ - 1u) / S_;                                   \
    const unsigned cost = rounds * (2u * (8u + 2u * RT_) * steps + (S_ > 1 ? 256u * RT_ : 0u));  \
    if (cost < best) {                                                                           \
      best = cost;                                                                               \
      p.rt = RT_;                                                                                \
      p.row_blocks = (int)rb;                                                                    \
      p.S = S_;                                                                                  \
    }                                                                                            \
  }
  VLAC_TALL_TRY(1, 4) VLAC_TALL_TRY(1, 3) VLAC_TALL_TRY(1, 2)
  VLAC_TALL_TRY(2, 4) VLAC_TALL_TRY(2, 3) VLAC_TALL_TRY(2, 2)
  VLAC_TALL_TRY(3, 4) VLAC_TALL_TRY(3, 3) VLAC_TALL_TRY(3, 2)
  VLAC_TALL_TRY(4, 4) VLAC_TALL_TRY(4, 3) VLAC_TALL_TRY(4, 2)
  VLAC_TALL_TRY(6, 4) VLAC_TALL_TRY(6, 3) VLAC_TALL_TRY(6, 2)
  VLAC_TALL_TRY(8, 4) VLAC_TALL_TRY(8, 3) VLAC_TALL_TRY(8, 2)
#undef VLAC_TALL_TRY
  return p;
}
// the same for the GEMM that launch_gemm(EPI_RESID, ...) with these arguments launches
SplitAdapt gemm_resid_adapt(vlac_ctx* c, int n_blocks, int kpad, int rows_cap, const int* n_rows, int n_rows_host);
int gemm_init();  // one-time kernel attribute setup; returns hipError_t
// returns the split-K factor used; for EPI_RESID a factor S > 1 means that the result is
// NOT in the residual stream yet but in e.rpart as S partial rows (more than 32 rows:
// always; at most 32 rows: if e.defer_split is set) for the consumer to add up
// (launch_resid_norm_rows, or NormIn::part of the next projection)
int launch_gemm(vlac_ctx* c, int epi, const bf16_t* wp, const float* wscale, int n_blocks, int kpad,
                const bf16_t* xp,
                 const int* n_rows, int n_rows_host, int rows_cap, const GemmEpi& e, hipStream_t st,
                 const NormIn* norm = nullptr);
// true if launch_gemm may be given a NormIn (RMSNorm fused into the GEMM)
bool gemm_can_fuse_norm(int n_rows_host, int decode_pos, int kpad);

// embed.hip
void launch_embed_patches(vlac_ctx* c, const uint8_t* frame, int B, int H, int W, int patch,
                          const bf16_t* w_proj, const int32_t* reuse_order, const int32_t* reuse_count,
                          int stride, const int32_t* layer_count, float* embeds, int L, hipStream_t st);

// attn.hip
// Text tiles per stream that the deferred statistic reduction provides for (text rows
// of a stream lie in at most ceil(L_t / 32) + 1 tiles: L_t <= 96).
static const int kStatDeferTT = 4;
// true if the attention kernels of a prefill only park their sums and
// launch_stats_reduce (once, after the last layer) writes out_attn_mean
bool attention_defers_stats(const vlac_ctx* c, int B, int L_v, int L_t);
void launch_stats_reduce(vlac_ctx* c, int B, int L_v, int L_t, float* out_attn_mean, hipStream_t st);
void launch_attention(vlac_ctx* c, int layer, int B, int rows_cap_per_stream, int L_v, int L_t,
                      const int* rows, const int* slot_off, int decode_pos, bf16_t* kv,
                      float* out_attn_mean, hipStream_t st);
