// Causal attention of the recomputed queries over the mixed KV cache, and the
// text-to-vision attention statistic (VLA-Cache appendix "Token Reuse
// Mechanism": newly computed tokens update their cache entries, reused tokens
// keep last step's, and attention over that partially updated cache is valid;
// Sec. 3.3, Eq. avistext for the statistic; Sec. 3.1 for the attention itself).
//
// A workgroup handles 32 query rows of one head; its 4 waves take every 4th tile
// of 32 cache positions (so a single decode query still spreads over 4 waves,
// and a head over its own workgroup), flash-style, entirely on the matrix cores,
// and merge their (max, sum, output) triples through LDS at the end:
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

struct AttnArgs {
  const int* rows;      // this layer's rows (b << 16 | pos)
  const int* slot_off;  // [B + 1] first slot of every stream
  int decode_pos;       // >= 0: one row per stream at this position; rows / slot_off are not read
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
  float* statp;         // [B][Hq][TT][lv_pad] (of this layer, if the reduction is deferred)
  int TT, lv_pad;
  int* stat_counters;   // [B]
  int defer_stats;      // the parked sums are added up by stats_reduce_kernel after the last layer
  int rows4_from;       // > 0: streams with at least this many rows are left to attn_rows4_kernel
  int dec_pack;         // decode with grouped queries: the query heads of one kv head share a workgroup
};

template <int HD, bool F16>
__global__ __launch_bounds__(256) void attn_rows_kernel(AttnArgs a) {
  constexpr int NC = HD / 16;  // k-tiles of a head
  constexpr int NI = HD / 32;  // feature blocks of a head
  __shared__ float cmb[3][2 + NI * 16][64];  // waves 1..3 park (max, sum, output) here
  __shared__ float fin[2][64];               // merged max and 1/sum per lane
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int j = lane & 31, g = lane >> 5;
  const int b = blockIdx.z;
  const bool dec = a.decode_pos >= 0;
  const int off_b = dec ? b : a.slot_off[b];
  const int n_b = dec ? 1 : a.slot_off[b + 1] - off_b;
  const int s0 = blockIdx.x * 32;
  if (s0 >= n_b) return;
  if (a.rows4_from > 0 && n_b >= a.rows4_from) return;
  // A decode pass has one query per stream and head, 1 column of the 32 a tile has.  With
  // grouped queries the heads that share a kv head fill the columns of ONE tile (blockIdx.y
  // is then the kv head, and the head is per lane): one workgroup per stream and kv head
  // reads the K and V tiles that group-many workgroups would each have read.
  const bool packed = dec && a.dec_pack;
  const int group = a.n_q_heads / a.n_kv_heads;
  const int hk = packed ? blockIdx.y : blockIdx.y / group;
  const int h = packed ? hk * group + min(j, group - 1) : blockIdx.y;
  const bool valid = packed ? j < group : s0 + j < n_b;
  const int sg = off_b + ((valid && !packed) ? s0 + j : n_b - 1);  // this lane's query slot
  const int pos = dec ? a.decode_pos : (valid ? (a.rows[sg] & 0xffff) : 0);
  const int pos_last = dec ? a.decode_pos : (a.rows[off_b + min(s0 + 31, n_b - 1)] & 0xffff);
  const int n_kt = (pos_last >> 5) + 1;

  const size_t head_elems = (size_t)a.max_seq * HD;
  const bf16_t* kbase = a.kv + (size_t)b * a.kv_stream_stride + (size_t)hk * head_elems +
                        (size_t)lane * 8;
  const bf16_t* vbase = kbase + (size_t)a.n_kv_heads * head_elems;

  uint4 qf[NC];
  {
    const bf16_t* qsrc = a.qbuf + ((size_t)(sg >> 5) * a.n_q_heads + h) * (size_t)NC * 512 +
                         (size_t)(((sg & 31) + 32 * g) << 3);
#pragma unroll
    for (int c = 0; c < NC; ++c) qf[c] = *(const uint4*)(qsrc + (size_t)c * 512);
  }
  auto load_k = [&](int kt, uint4(&kf)[NC]) {
#pragma unroll
    for (int c = 0; c < NC; ++c) kf[c] = *(const uint4*)(kbase + ((size_t)kt * NC + c) * 512);
  };
  auto scores = [&](const uint4(&kf)[NC], f32x16& s) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) s = mfma32<F16>(kf[c], qf[c], s);
  };

  f32x16 o[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ib][i] = 0.f;
  float m = -INFINITY, l = 0.f;

  uint4 kf[NC], kn[NC];
  if (w < n_kt) load_k(w, kf);
  for (int kt = w; kt < n_kt; kt += 4) {
    f32x16 s;
    scores(kf, s);
    uint4 vf[NI * 2];  // this tile's V, and the next tile's K, fly during the softmax arithmetic
#pragma unroll
    for (int t = 0; t < NI * 2; ++t) vf[t] = *(const uint4*)(vbase + ((size_t)kt * NI * 2 + t) * 512);
    if (kt + 4 < n_kt) load_k(kt + 4, kn);
    // register 4*q4 + e of a lane is key 32*kt + 8*q4 + 4*g + e
    float tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kp = 32 * kt + 8 * (i >> 2) + 4 * g + (i & 3);
      s[i] = (kp <= pos) ? s[i] * a.scale_log2e : -INFINITY;
      tmax = fmaxf(tmax, s[i]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    // a tile that lies wholly behind this query leaves max at -inf: keep the state as it is
    const float m_new = fmaxf(m, tmax);
    const float alpha = (m_new == -INFINITY) ? 1.f : exp2f(m - m_new);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    m = m_new;
    float psum = 0.f;
    float pr[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pr[i] = exp2f(s[i] - m_use);
      psum += pr[i];
    }
    l = l * alpha + psum;
    uint4 pb[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      pb[t].x = pack_op2<F16>(pr[8 * t + 0], pr[8 * t + 1]);
      pb[t].y = pack_op2<F16>(pr[8 * t + 2], pr[8 * t + 3]);
      pb[t].z = pack_op2<F16>(pr[8 * t + 4], pr[8 * t + 5]);
      pb[t].w = pack_op2<F16>(pr[8 * t + 6], pr[8 * t + 7]);
    }
#pragma unroll
    for (int ib = 0; ib < NI; ++ib) {
#pragma unroll
      for (int i = 0; i < 16; ++i) o[ib][i] *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t) o[ib] = mfma32<F16>(vf[ib * 2 + t], pb[t], o[ib]);
    }
#pragma unroll
    for (int c = 0; c < NC; ++c) kf[c] = kn[c];
  }
  l += __shfl_xor(l, 32);

  // merge the 4 waves (wave 0 owns tile 0, so its max is finite: key 0 is visible to every query)
  if (w > 0) {
    cmb[w - 1][0][lane] = m;
    cmb[w - 1][1][lane] = l;
#pragma unroll
    for (int ib = 0; ib < NI; ++ib)
#pragma unroll
      for (int i = 0; i < 16; ++i) cmb[w - 1][2 + ib * 16 + i][lane] = o[ib][i];
  }
  __syncthreads();
  if (w == 0) {
#pragma unroll
    for (int ww = 0; ww < 3; ++ww) {
      const float m_w = cmb[ww][0][lane], l_w = cmb[ww][1][lane];
      const float m_new = fmaxf(m, m_w);
      const float a0 = exp2f(m - m_new), a1 = exp2f(m_w - m_new);
      m = m_new;
      l = l * a0 + l_w * a1;
#pragma unroll
      for (int ib = 0; ib < NI; ++ib)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[ib][i] = o[ib][i] * a0 + cmb[ww][2 + ib * 16 + i][lane] * a1;
    }
    const float inv = 1.f / l;
    fin[0][lane] = m;
    fin[1][lane] = (valid && pos >= a.L_v) ? inv : 0.f;  // (the statistic counts text rows only)
    if (valid) {
#pragma unroll
      for (int ib = 0; ib < NI; ++ib)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int f = h * HD + 32 * ib + 8 * q4 + 4 * g;
          *(uint2*)(a.out + frag_off(sg, f, a.kc_out)) =
              make_uint2(pack_op2<F16>(o[ib][4 * q4] * inv, o[ib][4 * q4 + 1] * inv),
                         pack_op2<F16>(o[ib][4 * q4 + 2] * inv, o[ib][4 * q4 + 3] * inv));
        }
    }
  }

  // ---- text-to-vision statistic (all conditions are uniform over the workgroup) ----
  if (!a.attn_mean || a.L_t <= 0 || a.L_v <= 0 || dec) return;
  if (pos_last < a.L_v) return;  // no text row in this tile
  __syncthreads();
  const int x_first = (n_b - a.L_t) >> 5;  // first tile that holds a text row
  const int n_tt = ((n_b - 1) >> 5) - x_first + 1;
  const int tt = blockIdx.x - x_first;
  float* park = a.statp + (((size_t)b * a.n_q_heads + h) * a.TT + tt) * a.lv_pad;
  const int n_vt = (a.L_v + 31) >> 5;
  // Here the scores are taken the other way round, Q K^T: a lane's column is a KEY and its 16
  // registers are queries (8 q4 + 4 g + e, whose reference point and 1/sum wave 0 left in
  // LDS), so the sum over the queries of the tile is 16 additions in the lane and one
  // exchange between the two halves of the wave.
  const float* m_q = fin[0] + 4 * g;
  const float* inv_q = fin[1] + 4 * g;
  if (w < n_vt) load_k(w, kf);
  for (int kt = w; kt < n_vt; kt += 4) {
    f32x16 s;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) s = mfma32<F16>(qf[c], kf[c], s);
    if (kt + 4 < n_vt) load_k(kt + 4, kf);  // the next tile flies during the arithmetic
    float r = 0.f;  // fixed order: the lane's 16 queries, then the other half's
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int qi = 8 * (i >> 2) + (i & 3);
      const float iq = inv_q[qi];
      r += iq != 0.f ? exp2f(s[i] * a.scale_log2e - m_q[qi]) * iq : 0.f;
    }
    r += __shfl_xor(r, 32);
    if (g == 0) {
      if (a.defer_stats) park[32 * kt + j] = r;  // read by a later kernel: plain stores
      else st_coherent(park + 32 * kt + j, r);
    }
  }
  if (a.defer_stats) return;
  stores_done();
  __syncthreads();
  if (tid == 0) {
    const int expect = a.n_q_heads * n_tt;
    const int old = atomicAdd(a.stat_counters + b, 1);
    s_last = (old == expect - 1);
    if (old == expect - 1) a.stat_counters[b] = 0;
  }
  __syncthreads();
  if (!s_last) return;
  // the parked sums of all heads and text tiles, in fixed order, 16 loads in flight at a time
  const float norm = 1.f / ((float)a.n_q_heads * (float)a.L_t);
  const int n_part = a.n_q_heads * n_tt;
  const float* part0 = a.statp + (size_t)b * a.n_q_heads * a.TT * a.lv_pad;
  for (int v = tid; v < a.L_v; v += 256) {
    float acc = 0.f;
    for (int p0 = 0; p0 < n_part; p0 += 16) {
      float t[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = min(p0 + i, n_part - 1), hh = p / n_tt, tq = p - hh * n_tt;
        t[i] = ld_coherent(part0 + ((size_t)hh * a.TT + tq) * a.lv_pad + v);
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) acc += (p0 + i < n_part) ? t[i] : 0.f;
    }
    a.attn_mean[(size_t)b * a.attn_mean_stride + v] = acc * norm;
  }
}

// Two probabilities -> one operand dword.  They lie in [0, 256], so the fp16 conversion
// (round to nearest even, as everywhere) needs no saturation.
template <bool F16>
__device__ inline uint32_t pack_p2(float lo, float hi) {
  if constexpr (F16) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  } else {
    return pack_op2<false>(lo, hi);
  }
}

// ---------------------------------------------------------------------------
// The same attention for MANY query tiles per stream (long sequences, many streams): one
// query tile per WAVE.  The 4 waves of a workgroup walk the key tiles together and share
// every K and V tile through LDS (fragment order is kept, a tile is copied 16 bytes per
// thread as it lies), so a stream's cache is read once per 128 queries instead of once per
// 32, and there is nothing to merge.  A wave skips the key tiles behind its last query.
// The statistic is parked for stats_reduce_kernel (this kernel is only used where that
// reduction applies): waves that hold text rows run the second pass over the vision keys,
// whose K tiles the workgroup stages the same way.
// ---------------------------------------------------------------------------
// (3 waves per SIMD: measured 11 % faster than the 236 registers the compiler takes if allowed)
template <int HD, bool F16>
__global__ __launch_bounds__(256, 3) void attn_rows4_kernel(AttnArgs a) {
  constexpr int NC = HD / 16;      // k-tiles of a head
  constexpr int NI = HD / 32;      // feature blocks of a head
  constexpr int TILE = NC * 64;    // 16-byte chunks of a K tile (and of a V tile)
  constexpr int PER = TILE / 256;  // chunks per thread
  constexpr int AHEAD = 2;         // key tiles on their way to LDS while one is worked on (1 and 3: no faster)
  constexpr int NBUF = AHEAD + 1;
  __shared__ uint4 kvs[NBUF][2][TILE];  // [buffer][K, V]
  __shared__ int s_text[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int j = lane & 31, g = lane >> 5;
  // grid (heads, streams, query blocks): the query block is the slowest index, see below
  const int b = blockIdx.y, h = blockIdx.x;
  const int off_b = a.slot_off[b];
  const int n_b = a.slot_off[b + 1] - off_b;
  // the stream's query tiles are dealt to its workgroups in equal shares of at most 4 (33
  // tiles: 9 workgroups of 3 or 4, not 8 of 4 and one with a single busy wave)
  const int n_qt = (n_b + 31) >> 5, n_wg = (n_qt + 3) >> 2;
  if ((int)blockIdx.z >= n_wg || n_b < a.rows4_from) return;
  // The workgroups of the streams' LAST queries have the longest walks, and the launch lasts
  // as long as the last of them: they start first, those of ALL streams and heads before any
  // shorter one (the heads are the fastest index: workgroup id % 8, the XCD, is then the
  // same for all workgroups of a stream and head, which share its K and V in that L2).
  const int xb = n_wg - 1 - (int)blockIdx.z;
  const int qt_end = (xb + 1) * n_qt / n_wg;
  const int qt = xb * n_qt / n_wg + w, s0 = qt * 32;  // this wave's query tile
  const bool active = qt < qt_end;
  const int hk = h / (a.n_q_heads / a.n_kv_heads);
  const bool valid = active && s0 + j < n_b;
  const int sg = off_b + (valid ? s0 + j : n_b - 1);  // this lane's query slot
  const int pos = valid ? (a.rows[sg] & 0xffff) : 0;
  const int pos_last = active ? (a.rows[off_b + min(s0 + 31, n_b - 1)] & 0xffff) : -1;
  const int n_kt = (pos_last >> 5) + 1;  // 0 for a wave without queries
  const int pos_first = __builtin_amdgcn_readfirstlane(pos);  // lane 0: the wave's first query
  // rows ascend by position: the workgroup needs the key tiles of its last query
  const int pos_wg = a.rows[off_b + min(qt_end * 32 - 1, n_b - 1)] & 0xffff;
  const int n_kt_wg = (pos_wg >> 5) + 1;

  const size_t head_elems = (size_t)a.max_seq * HD;
  const uint4* ksrc = (const uint4*)(a.kv + (size_t)b * a.kv_stream_stride + (size_t)hk * head_elems) + tid;
  const uint4* vsrc = ksrc + (size_t)a.n_kv_heads * head_elems / 8;

  uint4 qf[NC];
  {
    const bf16_t* qsrc = a.qbuf + ((size_t)(sg >> 5) * a.n_q_heads + h) * (size_t)NC * 512 +
                         (size_t)(((sg & 31) + 32 * g) << 3);
#pragma unroll
    for (int c = 0; c < NC; ++c) qf[c] = *(const uint4*)(qsrc + (size_t)c * 512);
  }
  f32x16 o[NI];
#pragma unroll
  for (int ib = 0; ib < NI; ++ib)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ib][i] = 0.f;
  float m = -INFINITY, l = 0.f;

  // K and V tiles go global -> LDS directly (global_load_lds_dwordx4: lane l's 16 bytes
  // land at base + 16 l, so a wave copies 1 KiB as it lies), AHEAD tiles before they are
  // used, into a ring of AHEAD + 1 buffers: no staging registers, and the load latency is
  // spread over AHEAD tiles of work.  The copies are inline assembly, so the compiler does
  // not count them and the waits are placed by hand: loads return in issue order, every
  // tile is 2 PER copies per wave, nothing else is loaded inside the loop, and what was
  // loaded before it is older; so with the copies of AHEAD tiles issued, "at most
  // 2 PER (AHEAD - 1) outstanding" means that the oldest tile has landed.
  static_assert(PER == 1 || PER == 2, "a tile is 2 or 4 copies per wave");
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)&kvs[0][0][w * 64]);
  auto copy_tile = [&](int kt, int buf) {
    const uint4* ks = ksrc + (size_t)kt * TILE;
    const uint4* vs = vsrc + (size_t)kt * TILE;
    const uint32_t d = lds0 + buf * (2 * TILE * 16);
    if (PER == 2) {
      asm volatile(
          "s_mov_b32 m0, %0\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %4, off\n\t"
          "s_mov_b32 m0, %1\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %5, off\n\t"
          "s_mov_b32 m0, %2\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %6, off\n\t"
          "s_mov_b32 m0, %3\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %7, off"
          :
          : "s"(d), "s"(d + 4096), "s"(d + TILE * 16), "s"(d + TILE * 16 + 4096), "v"(ks), "v"(ks + 256),
            "v"(vs), "v"(vs + 256)
          : "memory", "m0");
    } else {
      asm volatile(
          "s_mov_b32 m0, %0\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %2, off\n\t"
          "s_mov_b32 m0, %1\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %3, off"
          :
          : "s"(d), "s"(d + TILE * 16), "v"(ks), "v"(vs)
          : "memory", "m0");
    }
  };
  // (the query fragments are waited for here, so that no wait for them ends up inside the loop,
  // where it would wait for the copies as well)
#pragma unroll
  for (int c = 0; c < NC; ++c) asm volatile("" ::"v"(qf[c].x), "v"(qf[c].y), "v"(qf[c].z), "v"(qf[c].w));
#pragma unroll
  for (int t = 0; t < AHEAD; ++t) copy_tile(min(t, n_kt_wg - 1), t);
  for (int kt = 0; kt < n_kt_wg; ++kt) {
    const int buf = kt % NBUF;
    // tile kt has landed (this wave's part; the barrier makes that all four parts), and every
    // wave has left tile kt - 1, whose buffer takes tile kt + AHEAD
    constexpr int YOUNGER = 2 * PER * (AHEAD - 1);
    static_assert(YOUNGER == 0 || YOUNGER == 2 || YOUNGER == 4 || YOUNGER == 8, "add the wait for this count");
    if (YOUNGER == 8) VLAC_VMCNT(8);
    else if (YOUNGER == 4) VLAC_VMCNT(4);
    else if (YOUNGER == 2) VLAC_VMCNT(2);
    else VLAC_VMCNT(0);
    __syncthreads();
    copy_tile(min(kt + AHEAD, n_kt_wg - 1), (kt + AHEAD) % NBUF);
    if (kt < n_kt) {
      f32x16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) s = mfma32<F16>(kvs[buf][0][c * 64 + lane], qf[c], s);
      // register 4*q4 + e of a lane is key 32*kt + 8*q4 + 4*g + e; only the tiles that
      // reach past the wave's first query need the causal mask
      float tmax = -INFINITY;
      if (32 * kt + 31 <= pos_first) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[i] *= a.scale_log2e;
          tmax = fmaxf(tmax, s[i]);
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int kp = 32 * kt + 8 * (i >> 2) + 4 * g + (i & 3);
          s[i] = (kp <= pos) ? s[i] * a.scale_log2e : -INFINITY;
          tmax = fmaxf(tmax, s[i]);
        }
      }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      // The reference point m of a query's exponentials follows its running maximum only
      // when that has grown by more than 8 (a factor of 256 in p, which fp16 operands and
      // fp32 sums hold easily): after the first tiles that is rare, and a tile in which no
      // query of the wave moves its reference skips the rescaling of the 64 accumulators.
      // (The decision is per query, so a query's result does not depend on its neighbours.)
      float alpha = 1.f;
      if (tmax > m + 8.f) {
        alpha = __builtin_amdgcn_exp2f(m - tmax);  // first tile: 2^-inf = 0
        m = tmax;
      }
      const float m_use = (m == -INFINITY) ? 0.f : m;
      float psum = 0.f;
      float pr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        pr[i] = __builtin_amdgcn_exp2f(s[i] - m_use);
        psum += pr[i];
      }
      l = l * alpha + psum;
      const bool rescale = __any(alpha != 1.f);
      uint4 pb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        pb[t].x = pack_p2<F16>(pr[8 * t + 0], pr[8 * t + 1]);
        pb[t].y = pack_p2<F16>(pr[8 * t + 2], pr[8 * t + 3]);
        pb[t].z = pack_p2<F16>(pr[8 * t + 4], pr[8 * t + 5]);
        pb[t].w = pack_p2<F16>(pr[8 * t + 6], pr[8 * t + 7]);
      }
      if (rescale) {
#pragma unroll
        for (int ib = 0; ib < NI; ++ib)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[ib][i] *= alpha;
      }
#pragma unroll
      for (int ib = 0; ib < NI; ++ib) {
#pragma unroll
        for (int t = 0; t < 2; ++t) o[ib] = mfma32<F16>(kvs[buf][1][(ib * 2 + t) * 64 + lane], pb[t], o[ib]);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no copy outlives the loop
  __syncthreads();                                  // (the buffers are used again below)
  l += __shfl_xor(l, 32);
  const float inv = 1.f / l;  // (a wave without queries: never used)
  if (valid) {
#pragma unroll
    for (int ib = 0; ib < NI; ++ib)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int f = h * HD + 32 * ib + 8 * q4 + 4 * g;
        *(uint2*)(a.out + frag_off(sg, f, a.kc_out)) =
            make_uint2(pack_op2<F16>(o[ib][4 * q4] * inv, o[ib][4 * q4 + 1] * inv),
                       pack_op2<F16>(o[ib][4 * q4 + 2] * inv, o[ib][4 * q4 + 3] * inv));
      }
  }

  // ---- text-to-vision statistic (the conditions up to the loop are uniform over the workgroup) ----
  if (!a.attn_mean || a.L_t <= 0 || a.L_v <= 0) return;
  if (pos_wg < a.L_v) return;  // no text row in this workgroup
  const int x_first = (n_b - a.L_t) >> 5;  // first query tile that holds a text row
  const bool text_wave = active && pos_last >= a.L_v;
  const bool is_text = valid && pos >= a.L_v;
  const int n_vt = (a.L_v + 31) >> 5;
  // The waves that hold text rows publish their query fragments, reference points and 1/sums
  // in LDS (all waves are past their last read of the buffers: the loop ended on a barrier);
  // then the 4 waves deal the vision key tiles of every such query tile among themselves,
  // each reading its K tiles straight from global memory: the workgroup with a stream's last
  // queries, which has the longest walk anyway, adds n_vt / 4 steps to it, not n_vt.
  uint4* q_sh = &kvs[0][0][0];                   // [4][NC][64]
  float* f_sh = (float*)(q_sh + 4 * NC * 64);    // [4][3][64]: reference point, 1/sum, text row?
  static_assert(4 * NC * 64 + 3 * 64 <= NBUF * 2 * TILE, "the buffers hold what the waves publish");
  if (text_wave) {
#pragma unroll
    for (int c = 0; c < NC; ++c) q_sh[(w * NC + c) * 64 + lane] = qf[c];
    f_sh[(w * 3 + 0) * 64 + lane] = m;
    f_sh[(w * 3 + 1) * 64 + lane] = is_text ? inv : 0.f;  // (a row that is no text row adds nothing)
    f_sh[(w * 3 + 2) * 64 + lane] = is_text ? 1.f : 0.f;
  }
  if (lane == 0) s_text[w] = text_wave ? 1 : 0;
  __syncthreads();
  const bf16_t* kbase = a.kv + (size_t)b * a.kv_stream_stride + (size_t)hk * head_elems + (size_t)lane * 8;
  auto load_k = [&](int kt, uint4(&kf)[NC]) {
#pragma unroll
    for (int c = 0; c < NC; ++c) kf[c] = *(const uint4*)(kbase + ((size_t)kt * NC + c) * 512);
  };
  // Here the scores are taken the other way round, Q K^T: a lane's column is a KEY and its 16
  // registers are queries (8 q4 + 4 g + e), so the sum over the queries of a tile is 16
  // additions in the lane and one exchange between the two halves of the wave.
  for (int tw = 0; tw < 4; ++tw) {
    if (!s_text[tw]) continue;
    uint4 qt_f[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) qt_f[c] = q_sh[(tw * NC + c) * 64 + lane];
    // per register: its query's reference point and 1/sum (0: no text row), read from LDS
    // where they are needed (they would cost 32 registers next to three K tiles)
    const float* m_q = f_sh + (tw * 3 + 0) * 64 + 4 * g;
    const float* inv_q = f_sh + (tw * 3 + 1) * 64 + 4 * g;
    float* park = a.statp + (((size_t)b * a.n_q_heads + h) * a.TT + (qt - w + tw - x_first)) * a.lv_pad;
    uint4 kf[NC], kn[NC];
    if (w < n_vt) load_k(w, kf);
    for (int kt = w; kt < n_vt; kt += 4) {
      if (kt + 4 < n_vt) load_k(kt + 4, kn);
      f32x16 s;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
      for (int c = 0; c < NC; ++c) s = mfma32<F16>(qt_f[c], kf[c], s);
      float r = 0.f;  // fixed order: the lane's 16 queries, then the other half's
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int qi = 8 * (i >> 2) + (i & 3);
        const float iq = inv_q[qi];
        r += iq != 0.f ? exp2f(s[i] * a.scale_log2e - m_q[qi]) * iq : 0.f;
      }
      r += __shfl_xor(r, 32);
      if (g == 0) park[32 * kt + j] = r;
#pragma unroll
      for (int c = 0; c < NC; ++c) kf[c] = kn[c];
    }
  }
}

// The statistic of all layers at once, after the last layer (text-to-vision attention
// averaged over heads and text queries, Eq. avistext): adds the sums that the attention
// kernels of the prefill parked, [layer][B][Hq][TT][lv_pad], over heads and text tiles in
// fixed order.  grid (layers, B); slot_off is [layers][slot_stride] (first slot of every
// stream at every layer), from which the number of text tiles follows as in the kernel.
__global__ __launch_bounds__(256) void stats_reduce_kernel(const float* __restrict__ statp,
                                                           const int* __restrict__ slot_off,
                                                           int slot_stride, int B, int n_q_heads,
                                                           int TT, int lv_pad, int L_v, int L_t,
                                                           float* __restrict__ attn_mean) {
  const int layer = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int* so = slot_off + (size_t)layer * slot_stride;
  const int n_b = so[b + 1] - so[b];
  const int x_first = (n_b - L_t) >> 5;
  const int n_tt = ((n_b - 1) >> 5) - x_first + 1;
  const int n_part = n_q_heads * n_tt;
  const float* part0 = statp + ((size_t)layer * B + b) * n_q_heads * TT * lv_pad;
  const float norm = 1.f / ((float)n_q_heads * (float)L_t);
  for (int v = tid; v < L_v; v += 256) {
    float acc = 0.f;
    for (int p0 = 0; p0 < n_part; p0 += 16) {
      float t[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = min(p0 + i, n_part - 1), hh = p / n_tt, tq = p - hh * n_tt;
        t[i] = part0[((size_t)hh * TT + tq) * lv_pad + v];
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) acc += (p0 + i < n_part) ? t[i] : 0.f;
    }
    attn_mean[((size_t)layer * B + b) * L_v + v] = acc * norm;
  }
}

bool attention_defers_stats(const vlac_ctx* c, int B, int L_v, int L_t) {
  // text rows of a stream lie in at most ceil(L_t / 32) + 1 tiles of 32 slots
  const int n_tt_max = (L_t + 31) / 32 + 1;
  const size_t need = (size_t)c->cfg.n_layers * B * c->cfg.n_q_heads * kStatDeferTT * round_up(L_v > 0 ? L_v : 1, 32);
  return L_t > 0 && L_v > 0 && n_tt_max <= kStatDeferTT && need <= c->statp_floats;
}

void launch_stats_reduce(vlac_ctx* c, int B, int L_v, int L_t, float* out_attn_mean, hipStream_t st) {
  hipLaunchKernelGGL(stats_reduce_kernel, dim3(c->cfg.n_layers, B), dim3(256), 0, st, c->statp,
                     c->slot_off, c->cfg.max_batch + 1, B, c->cfg.n_q_heads, kStatDeferTT,
                     round_up(L_v, 32), L_v, L_t, out_attn_mean);
}

void launch_attention(vlac_ctx* c, int layer, int B, int rows_cap_per_stream, int L_v, int L_t,
                      const int* rows, const int* slot_off, int decode_pos, bf16_t* kv,
                      float* out_attn_mean, hipStream_t st) {
  const vlac_model_cfg& m = c->cfg;
  AttnArgs a;
  a.rows = rows;
  a.slot_off = slot_off;
  a.decode_pos = decode_pos;
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
  a.lv_pad = round_up(L_v > 0 ? L_v : 1, 32);
  a.defer_stats = out_attn_mean && decode_pos < 0 && attention_defers_stats(c, B, L_v, L_t);
  if (a.defer_stats) {
    a.TT = kStatDeferTT;
    a.statp = c->statp + (size_t)layer * B * m.n_q_heads * kStatDeferTT * a.lv_pad;
  } else {
    a.TT = c->stat_tt;
    a.statp = c->statp;
  }
  a.stat_counters = c->stat_counters;
  // Sequences of 256 tokens or more of many streams (work for every CU several times over;
  // 32 streams x 304 tokens of the grouped-query model: 29.4 against 30.5 ms per full
  // prefill): streams with more
  // than two query tiles to recompute (65 rows) go to the kernel with one query tile per
  // WAVE, where the 4 waves of a workgroup share K and V (the cache is read once per 128
  // queries and not once per 32: measured at 8 streams x 1056 tokens, 134 rows per stream:
  // 4.2 ms per 32-layer prefill outside the GEMMs against 5.7 ms); streams with fewer rows
  // (and every other shape) to the kernel with one query tile per workgroup and the key
  // tiles dealt to its waves, which has the shorter critical path.  The row counts are
  // known on the device only, so both kernels are launched and each leaves the other's
  // streams alone.
  const int groups = (rows_cap_per_stream + 127) / 128;
  a.rows4_from = 0;
  if (decode_pos < 0 && rows_cap_per_stream >= 256 && (long long)groups * m.n_q_heads * B >= 512 &&
      (!a.attn_mean || a.defer_stats)) {
    a.rows4_from = 65;
    dim3 grid4(m.n_q_heads, B, groups);
    if (m.head_dim == 128) {
      if (c->f16) hipLaunchKernelGGL((attn_rows4_kernel<128, true>), grid4, dim3(256), 0, st, a);
      else hipLaunchKernelGGL((attn_rows4_kernel<128, false>), grid4, dim3(256), 0, st, a);
    } else {
      if (c->f16) hipLaunchKernelGGL((attn_rows4_kernel<64, true>), grid4, dim3(256), 0, st, a);
      else hipLaunchKernelGGL((attn_rows4_kernel<64, false>), grid4, dim3(256), 0, st, a);
    }
  }
  const int group = m.n_q_heads / m.n_kv_heads;
  a.dec_pack = decode_pos >= 0 && group > 1 && group <= 32;
  dim3 grid((rows_cap_per_stream + 31) / 32, a.dec_pack ? m.n_kv_heads : m.n_q_heads, B);
  if (m.head_dim == 128) {
    if (c->f16) hipLaunchKernelGGL((attn_rows_kernel<128, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_rows_kernel<128, false>), grid, dim3(256), 0, st, a);
  } else {
    if (c->f16) hipLaunchKernelGGL((attn_rows_kernel<64, true>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_rows_kernel<64, false>), grid, dim3(256), 0, st, a);
  }
}
