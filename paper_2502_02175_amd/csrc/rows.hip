// Row bookkeeping and the HBM-bound row kernels of the sparse prefill
// (Alg. 2 of VLA-Cache; appendix "Token Reuse Mechanism": the list of positions
// to recompute, recomputed rows keep their original positions).
//
//   plan_counts / plan_rows   per layer, the recomputed rows of every stream
//   rmsnorm_rows              gather a row of the residual stream, RMSNorm, write
//                             it as a bf16 matrix-core operand (fragment order)
//   final_hidden              final RMSNorm to fp32 (output)
//   argmax_rows, embed_rows   greedy token, token embedding lookup (decode)
//   pack_weights              weights -> fragment order (once per model)
#include "common.h"

// ---------------------------------------------------------------------------
// plan_counts: grid (B).  rank[b, v] = position of token v in stream b's reuse
// order (INT_MAX if it is not reusable); m_layer[b, l] = how many entries of the
// reuse order layer l reuses (clamped, non-decreasing over l);
// n_rows_bl[l, b] = rows stream b recomputes at layer l.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void plan_counts_kernel(
    int L_v, int L_t, int n_layers, int max_seq, const int32_t* __restrict__ reuse_order,
    const int32_t* __restrict__ reuse_count, int stride, const int32_t* __restrict__ layer_count,
    int* __restrict__ rank, int* __restrict__ m_layer, int* __restrict__ n_rows_bl, int B,
    int* __restrict__ errword) {
  __shared__ int red[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  int* rk = rank + (size_t)b * max_seq;
  for (int v = tid; v < L_v; v += 256) rk[v] = 0x7fffffff;
  __syncthreads();
  int cnt = 0;
  if (reuse_order && reuse_count) {
    cnt = reuse_count[b];
    if (cnt < 0 || cnt > stride) {
      if (tid == 0) atomicOr(errword, VLAC_ERR_BAD_INDEX);
      cnt = cnt < 0 ? 0 : stride;
    }
    for (int i = tid; i < cnt; i += 256) {
      const int v = reuse_order[(size_t)b * stride + i];
      if (v >= 0 && v < L_v) {
        const int old = atomicMin(&rk[v], i);
        if (old != 0x7fffffff) atomicOr(errword, VLAC_ERR_BAD_INDEX);  // repeated entry
      } else {
        atomicOr(errword, VLAC_ERR_BAD_INDEX);
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    int best = 0;
    for (int l = 0; l < n_layers; ++l) {
      int m = layer_count ? layer_count[(size_t)b * n_layers + l] : cnt;
      m = m < 0 ? 0 : (m > cnt ? cnt : m);
      best = m > best ? m : best;
      m_layer[(size_t)b * n_layers + l] = best;
    }
  }
  __syncthreads();
  for (int l = 0; l < n_layers; ++l) {
    const int m = m_layer[(size_t)b * n_layers + l];
    int n = 0;
    for (int v = tid; v < L_v; v += 256) n += rk[v] < m;
    for (int o = 32; o > 0; o >>= 1) n += __shfl_down(n, o);
    __syncthreads();
    if ((tid & 63) == 0) red[tid >> 6] = n;
    __syncthreads();
    if (tid == 0) n_rows_bl[(size_t)l * B + b] = L_v + L_t - (red[0] + red[1] + red[2] + red[3]);
  }
}

// plan_rows: grid (n_layers + 1, B).  Plane l < n_layers: rows of layer l, streams
// packed one after the other, positions ascending.  Plane n_layers: one row per
// stream, its last position (input of the output head).
__global__ __launch_bounds__(256) void plan_rows_kernel(
    int L_v, int L_t, int n_layers, int max_seq, int max_rows, int max_batch,
    const int* __restrict__ rank, const int* __restrict__ m_layer,
    const int* __restrict__ n_rows_bl, int B, int* __restrict__ rows, int* __restrict__ n_rows,
    int* __restrict__ slot_off, int* __restrict__ prev_slot) {
  __shared__ int wsum[4], wsum_p[4];
  __shared__ int base_s, base_p;
  const int l = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int L = L_v + L_t;
  if (l == n_layers) {
    if (tid == 0) {
      rows[(size_t)l * max_rows + b] = (b << 16) | (L - 1);
      slot_off[(size_t)l * (max_batch + 1) + b] = b;
      if (b == B - 1) {
        slot_off[(size_t)l * (max_batch + 1) + B] = B;
        n_rows[l] = B;
      }
    }
    return;
  }
  int off = 0, off_p = 0;  // first slot of this stream at this layer / at the layer before
  for (int k = 0; k < b; ++k) {
    off += n_rows_bl[(size_t)l * B + k];
    if (l > 0) off_p += n_rows_bl[(size_t)(l - 1) * B + k];
  }
  if (tid == 0) {
    slot_off[(size_t)l * (max_batch + 1) + b] = off;
    if (b == B - 1) {
      const int tot = off + n_rows_bl[(size_t)l * B + b];
      slot_off[(size_t)l * (max_batch + 1) + B] = tot;
      n_rows[l] = tot;
    }
    base_s = off;
    base_p = off_p;
  }
  __syncthreads();
  const int m = m_layer[(size_t)b * n_layers + l];
  const int m_p = l > 0 ? m_layer[(size_t)b * n_layers + l - 1] : 0;  // m is non-decreasing over l
  const int* rk = rank + (size_t)b * max_seq;
  for (int c0 = 0; c0 < L; c0 += 256) {
    const int p = c0 + tid;
    const int keep = p < L && !(p < L_v && rk[p] < m);
    const int keep_p = p < L && !(p < L_v && rk[p] < m_p);  // row of the layer before (a superset)
    const unsigned long long bal = __ballot(keep), bal_p = __ballot(keep_p);
    const unsigned long long below = (1ull << lane) - 1ull;
    const int inwave = __popcll(bal & below), inwave_p = __popcll(bal_p & below);
    if (lane == 0) { wsum[w] = __popcll(bal); wsum_p[w] = __popcll(bal_p); }
    __syncthreads();
    int o = base_s, o_p = base_p;
    for (int k = 0; k < w; ++k) { o += wsum[k]; o_p += wsum_p[k]; }
    if (keep) {
      rows[(size_t)l * max_rows + o + inwave] = (b << 16) | p;
      // where the same row sat in the previous layer's list (its FFN partial rows are there)
      prev_slot[(size_t)l * max_rows + o + inwave] = l > 0 ? o_p + inwave_p : o + inwave;
    }
    __syncthreads();
    if (tid == 0) {
      base_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
      base_p += wsum_p[0] + wsum_p[1] + wsum_p[2] + wsum_p[3];
    }
    __syncthreads();
  }
}

void launch_plan(vlac_ctx* c, int B, int L_v, int L_t, const int32_t* reuse_order,
                 const int32_t* reuse_count, int stride, const int32_t* layer_count,
                 hipStream_t st) {
  const int nl = c->cfg.n_layers;
  hipLaunchKernelGGL(plan_counts_kernel, dim3(B), dim3(256), 0, st, L_v, L_t, nl, c->cfg.max_seq,
                     reuse_order, reuse_count, stride, layer_count, c->rank, c->m_layer,
                     c->n_rows_bl, B, c->errword);
  hipLaunchKernelGGL(plan_rows_kernel, dim3(nl + 1, B), dim3(256), 0, st, L_v, L_t, nl,
                     c->cfg.max_seq, c->max_rows, c->cfg.max_batch, c->rank, c->m_layer,
                     c->n_rows_bl, B, c->rows, c->n_rows, c->slot_off, c->prev_slot);
}

// Decode row lists: plane t (0 <= t < n_new) holds row (b, L + t) for every stream.
__global__ void decode_plan_kernel(int B, int L, int n_new, int max_batch, int* __restrict__ rows,
                                   int* __restrict__ n_rows, int* __restrict__ slot_off) {
  const int t = blockIdx.x;
  for (int b = threadIdx.x; b <= B; b += blockDim.x) {
    if (b < B) rows[(size_t)t * max_batch + b] = (b << 16) | (L + t);
    slot_off[(size_t)t * (max_batch + 1) + b] = b;
  }
  if (threadIdx.x == 0) n_rows[t] = B;
}

void launch_decode_plan(vlac_ctx* c, int B, int L, int n_new, hipStream_t st) {
  // dec_rows layout: [n_new][max_batch] rows, then [n_new] counts, then [n_new][max_batch+1] offsets
  const int mb = c->cfg.max_batch, ms = c->cfg.max_seq;
  int* rows = c->dec_rows;
  int* n_rows = rows + (size_t)ms * mb;
  int* slot_off = n_rows + ms;
  hipLaunchKernelGGL(decode_plan_kernel, dim3(n_new), dim3(64), 0, st, B, L, n_new, mb, rows, n_rows,
                     slot_off);
}

// ---------------------------------------------------------------------------
// RMSNorm of the recomputed rows.  One wave per row: x * rsqrt(mean(x^2) + eps) * g,
// statistics in fp32, output bf16 in fragment order (slot = row of the operand).
// ---------------------------------------------------------------------------
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

template <bool F16>
__global__ __launch_bounds__(256) void rmsnorm_rows_kernel(
    const float* __restrict__ src, int seq_stride, const int* __restrict__ rows,
    const int* __restrict__ n_rows, int n_rows_host, int decode_pos,
    const float* __restrict__ gain, float eps, int d, bf16_t* __restrict__ xp, int KC) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (slot >= (n_rows_host >= 0 ? n_rows_host : *n_rows)) return;
  const int id = decode_pos >= 0 ? ((slot << 16) | decode_pos) : rows[slot];
  const float* x = src + ((size_t)(id >> 16) * seq_stride + (id & 0xffff)) * d;
  float ss = 0.f;
  for (int k = lane * 4; k < d; k += 256) {
    const float4 v = *(const float4*)(x + k);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  const float r = rsqrtf(ss / (float)d + eps);
  for (int k = lane * 8; k < d; k += 512) {
    const float4 a = *(const float4*)(x + k), b = *(const float4*)(x + k + 4);
    const float4 ga = *(const float4*)(gain + k), gb = *(const float4*)(gain + k + 4);
    uint4 o;
    o.x = pack_op2<F16>(a.x * r * ga.x, a.y * r * ga.y);
    o.y = pack_op2<F16>(a.z * r * ga.z, a.w * r * ga.w);
    o.z = pack_op2<F16>(b.x * r * gb.x, b.y * r * gb.y);
    o.w = pack_op2<F16>(b.z * r * gb.z, b.w * r * gb.w);
    *(uint4*)(xp + frag_off(slot, k, KC)) = o;
  }
}

// The same for rows of at most 512 NI elements: a lane keeps its share of the row (and of the
// gains) in registers, so every load of a row is in flight at once and the row is read once;
// with few rows (a decode pass over some streams) the kernel is all latency.
template <bool F16, int NI>
__global__ __launch_bounds__(256) void rmsnorm_rows_reg_kernel(
    const float* __restrict__ src, int seq_stride, const int* __restrict__ rows,
    const int* __restrict__ n_rows, int n_rows_host, int decode_pos,
    const float* __restrict__ gain, float eps, int d, bf16_t* __restrict__ xp, int KC) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (slot >= (n_rows_host >= 0 ? n_rows_host : *n_rows)) return;
  const int id = decode_pos >= 0 ? ((slot << 16) | decode_pos) : rows[slot];
  const float* x = src + ((size_t)(id >> 16) * seq_stride + (id & 0xffff)) * d;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 a[NI], b[NI], ga[NI], gb[NI];
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int k = lane * 8 + i * 512;
    a[i] = b[i] = ga[i] = gb[i] = zero;
    if (k < d) {
      a[i] = *(const float4*)(x + k);
      b[i] = *(const float4*)(x + k + 4);
      ga[i] = *(const float4*)(gain + k);
      gb[i] = *(const float4*)(gain + k + 4);
    }
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NI; ++i)
    ss += a[i].x * a[i].x + a[i].y * a[i].y + a[i].z * a[i].z + a[i].w * a[i].w +
          (b[i].x * b[i].x + b[i].y * b[i].y + b[i].z * b[i].z + b[i].w * b[i].w);
  ss = wave_sum(ss);
  const float r = rsqrtf(ss / (float)d + eps);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int k = lane * 8 + i * 512;
    if (k < d) {
      uint4 o;
      o.x = pack_op2<F16>(a[i].x * r * ga[i].x, a[i].y * r * ga[i].y);
      o.y = pack_op2<F16>(a[i].z * r * ga[i].z, a[i].w * r * ga[i].w);
      o.z = pack_op2<F16>(b[i].x * r * gb[i].x, b[i].y * r * gb[i].y);
      o.w = pack_op2<F16>(b[i].z * r * gb[i].z, b[i].w * r * gb[i].w);
      *(uint4*)(xp + frag_off(slot, k, KC)) = o;
    }
  }
}

void launch_rmsnorm_rows(bool f16, const float* src, int seq_stride, const int* rows,
                         const int* n_rows, int n_rows_host, int decode_pos, int max_rows,
                         const float* gain, float eps, int d, bf16_t* xp, int KC, hipStream_t st) {
  const dim3 grid((max_rows + 3) / 4), block(256);
#define VLAC_NORM_ARGS src, seq_stride, rows, n_rows, n_rows_host, decode_pos, gain, eps, d, xp, KC
  if (d <= 2048) {
    if (f16) hipLaunchKernelGGL((rmsnorm_rows_reg_kernel<true, 4>), grid, block, 0, st, VLAC_NORM_ARGS);
    else hipLaunchKernelGGL((rmsnorm_rows_reg_kernel<false, 4>), grid, block, 0, st, VLAC_NORM_ARGS);
  } else if (d <= 4096) {
    if (f16) hipLaunchKernelGGL((rmsnorm_rows_reg_kernel<true, 8>), grid, block, 0, st, VLAC_NORM_ARGS);
    else hipLaunchKernelGGL((rmsnorm_rows_reg_kernel<false, 8>), grid, block, 0, st, VLAC_NORM_ARGS);
  } else {
    if (f16) hipLaunchKernelGGL(rmsnorm_rows_kernel<true>, grid, block, 0, st, VLAC_NORM_ARGS);
    else hipLaunchKernelGGL(rmsnorm_rows_kernel<false>, grid, block, 0, st, VLAC_NORM_ARGS);
  }
#undef VLAC_NORM_ARGS
}

// Residual add with the split-K partial rows of the projection that came before, then
// (optionally) the RMSNorm that comes next: h[row] = resid[row] + sum_s part[s][slot]
// (in split order); xp[slot] = RMSNorm(h[row]) * gain.  One workgroup per row; the row
// stays in registers (MAXI float4 per thread, d <= 1024 * MAXI), and all of a thread's
// loads of the row and of two splits are in flight together: the work per row is all
// latency.  gain == nullptr: no norm.
template <bool F16, int MAXI, int NS>
__global__ __launch_bounds__(256) void resid_norm_rows_kernel(
    const float* __restrict__ resid, int resid_seq_stride, const float* __restrict__ part, int S,
    int part_rows, float* __restrict__ h, int h_seq_stride, const int* __restrict__ rows,
    const int* __restrict__ part_slot, const int* __restrict__ n_rows, int n_rows_host,
    const float* __restrict__ gain, float eps, int d, bf16_t* __restrict__ xp, int KC, SplitAdapt adapt) {
  __shared__ float red[4];
  const int slot = blockIdx.x, tid = threadIdx.x;
  if (slot >= (n_rows_host >= 0 ? n_rows_host : *n_rows)) return;
  const int id = rows[slot];
  // the partial rows are indexed by the slot the row had when the GEMM ran
  const int pslot = part_slot ? part_slot[slot] : slot;
  const float* r = resid + ((size_t)(id >> 16) * resid_seq_stride + (id & 0xffff)) * d;
  float* y = h + ((size_t)(id >> 16) * h_seq_stride + (id & 0xffff)) * d;
  if (adapt.n_blocks > 0) {
    // the GEMM chose its split factor from its row count; unsplit, it added to the
    // residual stream itself and left no partial rows
    const int n_g = adapt.n_rows_host >= 0 ? adapt.n_rows_host : *adapt.n_rows;
    S = n_g < adapt.small_below ? adapt.S_small : tall_plan((adapt.n_blocks + 7) >> 3, n_g, adapt.S_tall, adapt.KS).S;
    if (S == 1) {
      S = 0;
      r = y;
    }
  }
  const float* p0 = part + (size_t)pslot * d;
  const size_t pstride = (size_t)part_rows * d;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  // NS splits are in flight at a time (all 8 for rows of up to 4096 elements where the GEMM
  // may have split that far; 4 where it splits less, which leaves registers for more rows
  // per CU): a split past the last one is loaded from the last (a valid address, no branch)
  // and not added
  float4 v[MAXI], g[MAXI], t[NS][MAXI];
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    const int k = tid * 4 + i * 1024;
    v[i] = g[i] = zero;
    if (k < d) {
      v[i] = *(const float4*)(r + k);
      if (gain) g[i] = *(const float4*)(gain + k);
    }
  }
  for (int s = 0; s < S; s += NS) {  // fixed order
#pragma unroll
    for (int u = 0; u < NS; ++u)
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const int k = tid * 4 + i * 1024;
        t[u][i] = zero;
        if (k < d) t[u][i] = *(const float4*)(p0 + (size_t)min(s + u, S - 1) * pstride + k);
      }
#pragma unroll
    for (int u = 0; u < NS; ++u)
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const float on = s + u < S ? 1.f : 0.f;
        v[i].x += on * t[u][i].x; v[i].y += on * t[u][i].y;
        v[i].z += on * t[u][i].z; v[i].w += on * t[u][i].w;
      }
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    const int k = tid * 4 + i * 1024;
    if (k < d && (S > 0 || r != y)) *(float4*)(y + k) = v[i];  // (unsplit in place: h holds it already)
    ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
  }
  if (!gain) return;
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const float rinv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
#pragma unroll
  for (int i = 0; i < MAXI; ++i) {
    const int k = tid * 4 + i * 1024;
    if (k < d)
      *(uint2*)(xp + frag_off(slot, k, KC)) =
          make_uint2(pack_op2<F16>(v[i].x * rinv * g[i].x, v[i].y * rinv * g[i].y),
                     pack_op2<F16>(v[i].z * rinv * g[i].z, v[i].w * rinv * g[i].w));
  }
}

// Rows longer than 8192: the row is re-read instead of kept (a thread re-reads only what
// it wrote itself).
template <bool F16>
__global__ __launch_bounds__(256) void resid_norm_rows_long_kernel(
    const float* __restrict__ resid, int resid_seq_stride, const float* __restrict__ part, int S,
    int part_rows, float* __restrict__ h, int h_seq_stride, const int* __restrict__ rows,
    const int* __restrict__ part_slot, const int* __restrict__ n_rows, int n_rows_host,
    const float* __restrict__ gain, float eps, int d, bf16_t* __restrict__ xp, int KC) {
  __shared__ float red[4];
  const int slot = blockIdx.x, tid = threadIdx.x;
  if (slot >= (n_rows_host >= 0 ? n_rows_host : *n_rows)) return;
  const int id = rows[slot];
  const float* r = resid + ((size_t)(id >> 16) * resid_seq_stride + (id & 0xffff)) * d;
  float* y = h + ((size_t)(id >> 16) * h_seq_stride + (id & 0xffff)) * d;
  const float* p0 = part + (size_t)(part_slot ? part_slot[slot] : slot) * d;
  const size_t pstride = (size_t)part_rows * d;
  float ss = 0.f;
  for (int k = tid * 4; k < d; k += 1024) {
    float4 v = *(const float4*)(r + k);
    for (int s = 0; s < S; ++s) {  // fixed order
      const float4 q = *(const float4*)(p0 + (size_t)s * pstride + k);
      v.x += q.x; v.y += q.y; v.z += q.z; v.w += q.w;
    }
    *(float4*)(y + k) = v;
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  if (!gain) return;
  ss = wave_sum(ss);
  if ((tid & 63) == 0) red[tid >> 6] = ss;
  __syncthreads();
  const float rinv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
  for (int k = tid * 4; k < d; k += 1024) {
    const float4 v = *(const float4*)(y + k), g = *(const float4*)(gain + k);
    *(uint2*)(xp + frag_off(slot, k, KC)) =
        make_uint2(pack_op2<F16>(v.x * rinv * g.x, v.y * rinv * g.y),
                   pack_op2<F16>(v.z * rinv * g.z, v.w * rinv * g.w));
  }
}

void launch_resid_norm_rows(bool f16, const float* resid, int resid_seq_stride, const float* part,
                            int S, int part_rows, float* h, int h_seq_stride, const int* rows,
                            const int* part_slot, const int* n_rows, int n_rows_host, int max_rows,
                            const float* gain, float eps, int d, bf16_t* xp, int KC,
                            hipStream_t st, const SplitAdapt* adapt) {
  SplitAdapt ad = {nullptr, -1, 0, 0, 0, 0, 0};
  if (adapt) ad = *adapt;  // (never given for rows longer than 8192)
#define VLAC_RN(K)                                                                               \
  hipLaunchKernelGGL(K, dim3(max_rows), dim3(256), 0, st, resid, resid_seq_stride, part, S,      \
                     part_rows, h, h_seq_stride, rows, part_slot, n_rows, n_rows_host, gain, eps, \
                     d, xp, KC, ad)
  if (d <= 4096 && S <= 4) {
    if (f16) VLAC_RN((resid_norm_rows_kernel<true, 4, 4>));
    else VLAC_RN((resid_norm_rows_kernel<false, 4, 4>));
  } else if (d <= 4096) {
    if (f16) VLAC_RN((resid_norm_rows_kernel<true, 4, 8>));
    else VLAC_RN((resid_norm_rows_kernel<false, 4, 8>));
  } else if (d <= 8192) {
    if (f16) VLAC_RN((resid_norm_rows_kernel<true, 8, 4>));
    else VLAC_RN((resid_norm_rows_kernel<false, 8, 4>));
  } else {
#undef VLAC_RN
#define VLAC_RN(K)                                                                               \
  hipLaunchKernelGGL(K, dim3(max_rows), dim3(256), 0, st, resid, resid_seq_stride, part, S,      \
                     part_rows, h, h_seq_stride, rows, part_slot, n_rows, n_rows_host, gain, eps, \
                     d, xp, KC)
    if (f16) VLAC_RN(resid_norm_rows_long_kernel<true>);
    else VLAC_RN(resid_norm_rows_long_kernel<false>);
  }
#undef VLAC_RN
}

// Final RMSNorm of every row alive at the last layer, fp32 out [B, L, d].
__global__ __launch_bounds__(256) void final_hidden_kernel(
    const float* __restrict__ src, int seq_stride, const int* __restrict__ rows,
    const int* __restrict__ n_rows, const float* __restrict__ gain, float eps, int d,
    float* __restrict__ out, int L) {
  const int slot = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (slot >= *n_rows) return;
  const int id = rows[slot];
  const float* x = src + ((size_t)(id >> 16) * seq_stride + (id & 0xffff)) * d;
  float* y = out + ((size_t)(id >> 16) * L + (id & 0xffff)) * d;
  float ss = 0.f;
  for (int k = lane * 4; k < d; k += 256) {
    const float4 v = *(const float4*)(x + k);
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  const float r = rsqrtf(ss / (float)d + eps);
  for (int k = lane * 4; k < d; k += 256) {
    const float4 v = *(const float4*)(x + k), g = *(const float4*)(gain + k);
    *(float4*)(y + k) = make_float4(v.x * r * g.x, v.y * r * g.y, v.z * r * g.z, v.w * r * g.w);
  }
}

void launch_final_hidden(const float* src, int seq_stride, const int* rows, const int* n_rows,
                         int max_rows, const float* gain, float eps, int d, float* out, int L,
                         hipStream_t st) {
  hipLaunchKernelGGL(final_hidden_kernel, dim3((max_rows + 3) / 4), dim3(256), 0, st, src,
                     seq_stride, rows, n_rows, gain, eps, d, out, L);
}

// ---------------------------------------------------------------------------
// Greedy token: argmax over the vocabulary, ties -> lower id.  grid (B), 1024 threads.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits,
                                                      size_t logits_stride, int vocab,
                                                      int32_t* __restrict__ out, int out_stride,
                                                      int32_t* __restrict__ out2) {
  __shared__ float bv[16];
  __shared__ int bi[16];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* x = logits + (size_t)b * logits_stride;
  float best = -INFINITY;
  int idx = 0x7fffffff;
  auto take = [&](float v, int i) {
    if (v > best || (v == best && i < idx)) { best = v; idx = i; }
  };
  // 16-byte loads where the row allows them (base and stride multiples of 4 floats)
  const bool vec = ((((size_t)x) & 15) == 0);
  const int nv = vec ? (vocab & ~3) : 0;
  for (int i = tid * 4; i < nv; i += 4096) {
    const float4 v = *(const float4*)(x + i);
    take(v.x, i); take(v.y, i + 1); take(v.z, i + 2); take(v.w, i + 3);
  }
  for (int i = nv + tid; i < vocab; i += 1024) take(x[i], i);
  for (int o = 32; o > 0; o >>= 1) {
    const float v = __shfl_xor(best, o);
    const int i = __shfl_xor(idx, o);
    take(v, i);
  }
  if ((tid & 63) == 0) { bv[tid >> 6] = best; bi[tid >> 6] = idx; }
  __syncthreads();
  if (tid == 0) {
    for (int k = 1; k < 16; ++k) take(bv[k], bi[k]);
    if (idx == 0x7fffffff) idx = 0;  // every logit NaN: still a valid id
    out[(size_t)b * out_stride] = idx;
    if (out2) out2[b] = idx;
  }
}

void launch_argmax(const float* logits, size_t logits_stride, int B, int vocab, int32_t* out,
                   int out_stride, int32_t* out2, hipStream_t st) {
  hipLaunchKernelGGL(argmax_kernel, dim3(B), dim3(1024), 0, st, logits, logits_stride, vocab, out,
                     out_stride, out2);
}

// Token embedding rows into the residual stream at position `pos`.  grid (B).
__global__ __launch_bounds__(256) void embed_rows_kernel(const bf16_t* __restrict__ embed,
                                                         const int32_t* __restrict__ tokens, int d,
                                                         int vocab, float* __restrict__ h,
                                                         int max_seq, int pos) {
  const int b = blockIdx.x;
  int tok = tokens[b];
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);
  const bf16_t* e = embed + (size_t)tok * d;
  float* y = h + ((size_t)b * max_seq + pos) * d;
  for (int k = threadIdx.x; k < d; k += 256) y[k] = __uint_as_float((uint32_t)e[k] << 16);
}

void launch_embed_rows(const bf16_t* embed, const int32_t* tokens, int B, int d, int vocab, float* h,
                       int max_seq, int pos, hipStream_t st) {
  hipLaunchKernelGGL(embed_rows_kernel, dim3(B), dim3(256), 0, st, embed, tokens, d, vocab, h,
                     max_seq, pos);
}

// ---------------------------------------------------------------------------
// Weights [N, K] row-major -> fragment order, with a row permutation:
//   mode 0  identity
//   mode 1  QKV (p0 = Hq*hd, p1 = Hkv*hd, p2 = hd): inside every 32-row block of a
//           query or key head the two rotary partners (f, f + hd/2) of 16
//           features sit 16 rows apart, so one lane of the GEMM epilogue holds
//           both; value heads keep their order
//   mode 2  gate/up (p0 = F): every 32-row block holds 16 gate rows followed by
//           the 16 matching up rows
// Rows >= n_pack sources and columns >= K are zero.  With to_f16 the bf16 values are
// re-encoded as fp16 (exact but for magnitudes below 2^-14, which round to
// multiples of 2^-24).
// ---------------------------------------------------------------------------
__device__ inline int pack_src_row(int pr, int mode, int p0, int p1, int p2) {
  if (mode == 1) {
    if (pr >= p0 + p1) return pr;
    const int hd = p2, within = pr % hd, sb = within >> 5, i = within & 31;
    const int f = (i < 16) ? 16 * sb + i : hd / 2 + 16 * sb + (i - 16);
    return pr - within + f;
  }
  if (mode == 2) {
    const int blk = pr >> 5, i = pr & 31;
    return (i < 16) ? 16 * blk + i : p0 + 16 * blk + (i - 16);
  }
  return pr;
}

__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t* __restrict__ src, int N,
                                                           int K, bf16_t* __restrict__ dst,
                                                           int n_pack, int kpad, int mode, int p0,
                                                           int p1, int p2, int to_f16) {
  const int KC = kpad / 16;
  const size_t n_chunks = (size_t)(n_pack / 32) * KC * 64;  // 16-byte chunks
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < n_chunks;
       c += (size_t)gridDim.x * 256) {
    const int lane = (int)(c & 63);
    const size_t tile = c >> 6;
    const int kc = (int)(tile % KC), rt = (int)(tile / KC);
    const int pr = rt * 32 + (lane & 31), col = kc * 16 + 8 * (lane >> 5);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (col < K) {
      const int sr = pack_src_row(pr, mode, p0, p1, p2);
      if (sr < N) v = *(const uint4*)(src + (size_t)sr * K + col);
      if (to_f16) {  // bf16 -> fp32 (exact) -> fp16
        uint32_t* u = (uint32_t*)&v;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          u[i] = pack_op2<true>(__uint_as_float(u[i] << 16), __uint_as_float(u[i] & 0xffff0000u));
      }
    }
    *(uint4*)(dst + c * 8) = v;
  }
}

void launch_pack(bool to_f16, const bf16_t* src, int N, int K, bf16_t* dst, int n_pack, int kpad,
                 int mode, int p0, int p1, int p2, hipStream_t st) {
  hipLaunchKernelGGL(pack_weights_kernel, dim3(2048), dim3(256), 0, st, src, N, K, dst, n_pack,
                     kpad, mode, p0, p1, p2, to_f16 ? 1 : 0);
}

// ---------------------------------------------------------------------------
// Weight-only e4m3 storage.  Scale of a row: the smallest power of two s with
// max|w_row| / s <= 448 (the largest e4m3 value), 1 for a zero row, never below 2^-120.
// Codes: round to nearest representable value, ties to the even mantissa.
// ---------------------------------------------------------------------------
__device__ inline float bf16_val(bf16_t x) { return __uint_as_float((uint32_t)x << 16); }
// 1 / s for a power of two s, by its exponent field
__device__ inline float pow2_inverse(float s) { return __uint_as_float((254u - (__float_as_uint(s) >> 23)) << 23); }

// OCP e4m3 code of x, |x| <= 448: below the smallest normal 2^-6 the values are the
// multiples of 2^-9 (rintf rounds to nearest even); above, the fp32 mantissa is rounded
// to 3 bits in the integer domain, which carries into the exponent by itself.
__device__ inline uint32_t e4m3_encode(float x) {
  const uint32_t sign = (__float_as_uint(x) >> 24) & 0x80u;
  const float a = fabsf(x);
  uint32_t code;
  if (a < 0.015625f) {
    code = (uint32_t)rintf(a * 512.f);  // 0 .. 8; 8 is the code of 2^-6
  } else {
    uint32_t v = __float_as_uint(a);
    v += 0x7ffffu + ((v >> 20) & 1u);
    code = (v >> 20) - ((127u - 7u) << 3);  // (exponent field - 120) << 3 | mantissa
    if (code > 126u) code = 126u;
  }
  return code | sign;
}

__global__ __launch_bounds__(256) void row_scales_kernel(const bf16_t* __restrict__ src, int N, int K,
                                                         float* __restrict__ scales) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= N) return;
  float m = 0.f;
  for (int k = lane; k < K; k += 64) m = fmaxf(m, fabsf(bf16_val(src[(size_t)row * K + k])));
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if (lane == 0) {
    float s = 1.f;
    if (m > 0.f) {
      // m = f * 2^E, 1 <= f < 2:  f * 2^(E - e) <= 1.75 * 2^8  <=>  e >= E - 8 (f <= 1.75) or E - 7
      const uint32_t u = __float_as_uint(m);
      int E = (int)(u >> 23) - 127;
      const uint32_t frac = u & 0x7fffffu;
      if ((u >> 23) == 0) E = -127;  // (fp32 subnormal: far below the floor anyway)
      int e = E - 8 + (frac > 0x600000u ? 1 : 0);  // 0x600000 = .75
      if (e < -120) e = -120;
      s = __uint_as_float((uint32_t)(e + 127) << 23);
    }
    scales[row] = s;
  }
}

void launch_row_scales(const bf16_t* src, int N, int K, float* scales, hipStream_t st) {
  hipLaunchKernelGGL(row_scales_kernel, dim3((N + 3) / 4), dim3(256), 0, st, src, N, K, scales);
}

__global__ __launch_bounds__(256) void quantize_e4m3_kernel(const bf16_t* __restrict__ src, int N, int K,
                                                            const float* __restrict__ scales,
                                                            uint8_t* __restrict__ codes) {
  const size_t n = (size_t)N * K;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const float inv = pow2_inverse(scales[i / K]);
    codes[i] = (uint8_t)e4m3_encode(bf16_val(src[i]) * inv);
  }
}

void launch_quantize_e4m3(const bf16_t* src, int N, int K, const float* scales, uint8_t* codes,
                          hipStream_t st) {
  hipLaunchKernelGGL(quantize_e4m3_kernel, dim3(1024), dim3(256), 0, st, src, N, K, scales, codes);
}

// Codes in fragment order: a 16-byte lane slot holds the lane's 8 codes of k-tile 2c and
// its 8 codes of k-tile 2c + 1 (lane = (row % 32) + 32 * ((col % 16) / 8) as for the 16-bit
// operands), so one 1 KiB wave load brings two k-tiles.  Row permutation as pack_weights_kernel.
__global__ __launch_bounds__(256) void pack_e4m3_kernel(const bf16_t* __restrict__ src, int N, int K,
                                                        const float* __restrict__ scales,
                                                        bf16_t* __restrict__ dst, float* __restrict__ scales_packed,
                                                        int n_pack, int kpad, int mode, int p0, int p1, int p2) {
  const int KC2 = kpad / 32;
  const size_t n_chunks = (size_t)(n_pack / 32) * KC2 * 64;  // 16-byte chunks
  for (size_t c = (size_t)blockIdx.x * 256 + threadIdx.x; c < n_chunks; c += (size_t)gridDim.x * 256) {
    const int lane = (int)(c & 63);
    const size_t tile = c >> 6;
    const int kc2 = (int)(tile % KC2), rt = (int)(tile / KC2);
    const int pr = rt * 32 + (lane & 31);
    const int sr = pack_src_row(pr, mode, p0, p1, p2);
    uint32_t out[4] = {0, 0, 0, 0};
    if (sr < N) {
      const float inv = pow2_inverse(scales[sr]);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int col = (2 * kc2 + h) * 16 + 8 * (lane >> 5);
        if (col < K) {  // K is a multiple of 8
          const uint4 v = *(const uint4*)(src + (size_t)sr * K + col);
          const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const uint32_t lo = e4m3_encode(__uint_as_float(u[i] << 16) * inv);
            const uint32_t hi = e4m3_encode(__uint_as_float(u[i] & 0xffff0000u) * inv);
            out[2 * h + (i >> 1)] |= (lo | (hi << 8)) << (16 * (i & 1));
          }
        }
      }
    }
    *(uint4*)((char*)dst + c * 16) = make_uint4(out[0], out[1], out[2], out[3]);
    if (kc2 == 0 && lane < 32) scales_packed[pr] = sr < N ? scales[sr] : 1.f;
  }
}

void launch_pack_e4m3(const bf16_t* src, int N, int K, const float* scales, bf16_t* dst, float* scales_packed,
                      int n_pack, int kpad, int mode, int p0, int p1, int p2, hipStream_t st) {
  hipLaunchKernelGGL(pack_e4m3_kernel, dim3(2048), dim3(256), 0, st, src, N, K, scales, dst, scales_packed,
                     n_pack, kpad, mode, p0, p1, p2);
}

__global__ void bf16_to_f32_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = __uint_as_float((uint32_t)src[i] << 16);
}

void launch_bf16_to_f32(const bf16_t* src, float* dst, int n, hipStream_t st) {
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, n);
}
