// Causal attention of the recomputed queries over the mixed KV cache, and the
// text-to-vision attention statistic (VLA-Cache appendix "Token Reuse
// Mechanism": newly computed tokens update their cache entries, reused tokens
// keep last step's, and attention over that partially updated cache is valid;
// Sec. 3.3, Eq. avistext for the statistic; Sec. 3.1 for the attention itself).
//
// One wave handles 32 query rows of one head, flash-style over tiles of 32 cache
// positions, entirely on the matrix cores and without LDS:
//   S^T[key, query] = K . Q^T   A operand: K tile (fragment order in the cache),
//                               B operand: Q tile (fragment order from the QKV epilogue)
//   O^T[feat, query] += V^T . P^T  A operand: V tile (the cache stores V per 32
//                               positions already transposed and in the key order
//                               in which a lane holds its scores), B operand: P
// so a lane owns one query column throughout: the running max / sum are
// per-lane scalars (one exchange between the two half-waves per tile) and P goes
// from the score registers straight into the next MFMA.
// Rows are the recomputed rows of the layer, sorted by position inside each
// stream; a query at position p sees cache positions 0..p, fresh or reused.
//
// Statistic: waves whose tile holds text queries run a second pass over the
// vision keys with the final max/sum, sum the probabilities over their text
// rows, and park the sums; the last workgroup of a stream to arrive (atomic
// counter, no waiting) adds the parked sums over heads and tiles in fixed order.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct AttnArgs {
  const int* rows;      // this layer's rows (b << 16 | pos)
  const int* slot_off;  // [B + 1] first slot of every stream
  const bf16_t* qbuf;
  bf16_t* out;          // attention output, fragment order, KC = kc_out
  int kc_out;
  const bf16_t* kv;     // cache base (stream 0) of this layer
  size_t kv_stream_stride;
  int n_q_heads, n_kv_heads, max_seq;
  int L_v, L_t;
  float scale_log2e;    // log2(e) / sqrt(head_dim)
  float* attn_mean;     // [B, L_v] of this layer or NULL
  int attn_mean_stride; // elements between streams
  float* statp;         // [B][Hq][TT][lv_pad]
  int TT, lv_pad;
  int* stat_counters;   // [B]
};

template <int HD>
__global__ __launch_bounds__(256) void attn_rows_kernel(AttnArgs a) {
  constexpr int NC = HD / 16;  // k-tiles of a head
  constexpr int NI = HD / 32;  // feature blocks of a head
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int j = lane & 31, g = lane >> 5;
  const int b = blockIdx.z, h = blockIdx.y * 4 + w;
  const int off_b = a.slot_off[b], n_b = a.slot_off[b + 1] - off_b;
  const int s0 = blockIdx.x * 32;
  if (s0 >= n_b) return;
  const int hk = h / (a.n_q_heads / a.n_kv_heads);
  const bool valid = s0 + j < n_b;
  const int sg = off_b + (valid ? s0 + j : n_b - 1);  // this lane's query slot
  const int pos = valid ? (a.rows[sg] & 0xffff) : 0;
  const int pos_last = a.rows[off_b + min(s0 + 31, n_b - 1)] & 0xffff;
  const int n_kt = (pos_last >> 5) + 1;

  const size_t head_elems = (size_t)a.max_seq * HD;
  const bf16_t* kbase = a.kv + (size_t)b * a.kv_stream_stride + (size_t)hk * head_elems;
  const bf16_t* vbase = kbase + (size_t)a.n_kv_heads * head_elems;

  bf16x8 qf[NC];
  {
    const bf16_t* qsrc = a.qbuf + ((size_t)(sg >> 5) * a.n_q_heads + h) * (size_t)NC * 512 +
                         (size_t)(((sg & 31) + 32 * g) << 3);
#pragma unroll
    for (int c = 0; c < NC; ++c) qf[c] = *(const bf16x8*)(qsrc + (size_t)c * 512);
  }

  auto scores = [&](int kt, f32x16& s) {
    const bf16_t* kt_base = kbase + (size_t)kt * NC * 512 + (size_t)lane * 8;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const bf16x8 kf = *(const bf16x8*)(kt_base + (size_t)c * 512);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[c], s, 0, 0, 0);
    }
  };

  f32x16 o[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ib][i] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int kt = 0; kt < n_kt; ++kt) {
    f32x16 s;
    scores(kt, s);
    // register 4*q4 + e of a lane is key 32*kt + 8*q4 + 4*g + e
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kp = 32 * kt + 8 * (i >> 2) + 4 * g + (i & 3);
      s[i] = (kp <= pos) ? s[i] * a.scale_log2e : -INFINITY;
      tmax = fmaxf(tmax, s[i]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_new = fmaxf(m, tmax);  // finite from tile 0 on: key 0 is visible to every query
    const float alpha = exp2f(m - m_new);
    m = m_new;
    float psum = 0.f;
    float p[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      p[i] = exp2f(s[i] - m_new);
      psum += p[i];
    }
    l = l * alpha + psum;
    bf16x8 pb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint4 u;
      u.x = pack_bf16x2(p[8 * t + 0], p[8 * t + 1]);
      u.y = pack_bf16x2(p[8 * t + 2], p[8 * t + 3]);
      u.z = pack_bf16x2(p[8 * t + 4], p[8 * t + 5]);
      u.w = pack_bf16x2(p[8 * t + 6], p[8 * t + 7]);
      pb[t] = __builtin_bit_cast(bf16x8, u);
    }
    const bf16_t* vt_base = vbase + (size_t)kt * NI * 2 * 512 + (size_t)lane * 8;
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
#pragma unroll
      for (int i = 0; i < 16; ++i) o[ib][i] *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8 vf = *(const bf16x8*)(vt_base + (size_t)(ib * 2 + t) * 512);
        o[ib] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[t], o[ib], 0, 0, 0);
      }
    }
  }
  l += __shfl_xor(l, 32);
  const float inv = 1.f / l;

  if (valid) {
#pragma unroll
    for (int ib = 0; ib < NI; ++ib)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int f = h * HD + 32 * ib + 8 * q4 + 4 * g;
        *(uint2*)(a.out + frag_off(sg, f, a.kc_out)) =
            make_uint2(pack_bf16x2(o[ib][4 * q4] * inv, o[ib][4 * q4 + 1] * inv),
                       pack_bf16x2(o[ib][4 * q4 + 2] * inv, o[ib][4 * q4 + 3] * inv));
      }
  }

  // ---- text-to-vision statistic ----
  if (!a.attn_mean || a.L_t <= 0 || a.L_v <= 0) return;
  if (pos_last < a.L_v) return;  // no text row in this tile (uniform over the workgroup)
  const int x_first = (n_b - a.L_t) >> 5;  // first tile that holds a text row
  const int n_tt = ((n_b - 1) >> 5) - x_first + 1;
  const int tt = blockIdx.x - x_first;
  const bool is_text = valid && pos >= a.L_v;
  float* park = a.statp + (((size_t)b * a.n_q_heads + h) * a.TT + tt) * a.lv_pad;
  const int n_vt = (a.L_v + 31) >> 5;
  for (int kt = 0; kt < n_vt; ++kt) {
    f32x16 s;
    scores(kt, s);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float pv = is_text ? exp2f(s[i] * a.scale_log2e - m) * inv : 0.f;
      // sum over the 32 queries of the tile (the lanes of a half-wave), fixed order
#pragma unroll
      for (int d = 1; d < 32; d <<= 1) pv += __shfl_xor(pv, d);
      s[i] = pv;
    }
    if (j == 0) {
#pragma unroll
      for (int i = 0; i < 16; ++i) park[32 * kt + 8 * (i >> 2) + 4 * g + (i & 3)] = s[i];
    }
  }
  __threadfence();
  __syncthreads();
  if (tid == 0) {
    const int expect = (a.n_q_heads / 4) * n_tt;
    const int old = atomicAdd(a.stat_counters + b, 1);
    s_last = (old == expect - 1);
    if (old == expect - 1) a.stat_counters[b] = 0;
  }
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  const float norm = 1.f / ((float)a.n_q_heads * (float)a.L_t);
  for (int v = tid; v < a.L_v; v += 256) {
    float acc = 0.f;
    for (int hh = 0; hh < a.n_q_heads; ++hh)
      for (int t = 0; t < n_tt; ++t)
        acc += a.statp[(((size_t)b * a.n_q_heads + hh) * a.TT + t) * a.lv_pad + v];
    a.attn_mean[(size_t)b * a.attn_mean_stride + v] = acc * norm;
  }
}

void launch_attention(vlac_ctx* c, int layer, int B, int rows_cap_per_stream, int L_v, int L_t,
                      const int* rows, const int* slot_off, bf16_t* kv, float* out_attn_mean,
                      hipStream_t st) {
  const vlac_model_cfg& m = c->cfg;
  AttnArgs a;
  a.rows = rows;
  a.slot_off = slot_off;
  a.qbuf = c->qbuf;
  a.out = c->xa;
  a.kc_out = c->kpad_q / 16;
  const size_t layer_elems = (size_t)2 * m.n_kv_heads * m.max_seq * m.head_dim;
  a.kv = kv + (size_t)layer * layer_elems;
  a.kv_stream_stride = (size_t)m.n_layers * layer_elems;
  a.n_q_heads = m.n_q_heads;
  a.n_kv_heads = m.n_kv_heads;
  a.max_seq = m.max_seq;
  a.L_v = L_v;
  a.L_t = L_t;
  a.scale_log2e = 1.4426950408889634f / sqrtf((float)m.head_dim);
  a.attn_mean = out_attn_mean ? out_attn_mean + (size_t)layer * B * L_v : nullptr;
  a.attn_mean_stride = L_v;
  a.statp = c->statp;
  a.TT = c->stat_tt;
  a.lv_pad = round_up(L_v > 0 ? L_v : 1, 32);
  a.stat_counters = c->stat_counters;
  dim3 grid((rows_cap_per_stream + 31) / 32, m.n_q_heads / 4, B);
  if (m.head_dim == 128)
    hipLaunchKernelGGL(attn_rows_kernel<128>, grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL(attn_rows_kernel<64>, grid, dim3(256), 0, st, a);
}
