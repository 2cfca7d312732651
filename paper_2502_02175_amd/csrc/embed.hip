// Front end for the visual tokens: the patch -> embedding projection, for the patches
// that the sparse prefill will recompute only (an extension of the token reuse of
// VLA-Cache, Sec. 3.2 / Alg. 2, to the step before the decoder: a token whose K/V are
// reused at the first layer needs no embedding either).  The projection is a fixed linear
// map of the patch's pixels, the stand-in used here for the vision encoder:
//   e[i, :] = (pixels_i / 127.5 - 1) . W,   pixels_i = patch i as [p rows][p cols][3] bytes.
//
// Work: (changed patches) x 3 p^2 x d multiply-adds against a matrix of a few MB that stays
// in L2: plain fp32 FMAs, 8 patches per workgroup so that a weight is loaded once per 8
// products; pixels are staged in LDS as fp32.  The patches to do are compacted into a list
// first, so that the work is proportional to their number.
#include "common.h"

// list[b][0 .. n_live[b]) = the patches of stream b that are NOT among the first m reuse
// entries, ascending.  One workgroup per stream.
__global__ __launch_bounds__(256) void embed_mark_kernel(const int32_t* __restrict__ reuse_order,
                                                         const int32_t* __restrict__ reuse_count,
                                                         int stride, const int32_t* __restrict__ layer_count,
                                                         int n_layers, int L_v, uint8_t* __restrict__ flags,
                                                         int* __restrict__ list, int* __restrict__ n_live) {
  __shared__ int wsum[4];
  __shared__ int base;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  uint8_t* f = flags + (size_t)b * 4096;
  int* out = list + (size_t)b * 4096;
  for (int i = tid; i < L_v; i += 256) f[i] = 0;
  __syncthreads();
  if (reuse_order) {
    int m = min(max(reuse_count[b], 0), stride);
    if (layer_count) m = min(m, max(layer_count[(size_t)b * n_layers], 0));
    for (int i = tid; i < m; i += 256) {
      const int t = reuse_order[(size_t)b * stride + i];
      if (t >= 0 && t < L_v) f[t] = 1;
    }
  }
  if (tid == 0) base = 0;
  __syncthreads();
  for (int i0 = 0; i0 < L_v; i0 += 256) {  // ordered compaction, 256 patches at a time
    const int i = i0 + tid;
    const bool live = i < L_v && !f[i];
    const unsigned long long mask = __ballot(live);
    if (lane == 0) wsum[w] = __popcll(mask);
    __syncthreads();
    int off = base;
    for (int k = 0; k < w; ++k) off += wsum[k];
    if (live) out[off + __popcll(mask & ((1ull << lane) - 1))] = i;
    __syncthreads();
    if (tid == 0) base += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
  if (tid == 0) n_live[b] = base;
}

constexpr int EMB_PB = 8;   // patches per workgroup
constexpr int EMB_CH = 12;  // values of k per batch of weight loads

// Workgroup (x: 256 output features, y: group of 8 live patches, z: stream).  Pixels of the
// group go to LDS as fp32 [k][8 patches], so that a thread fetches the 8 values of one k
// with two 16-byte reads (all lanes the same address) and does 8 multiply-adds per weight.
__global__ __launch_bounds__(256) void embed_patches_kernel(const uint8_t* __restrict__ frame, int H, int W,
                                                            int patch, const bf16_t* __restrict__ w_proj,
                                                            int d, const int* __restrict__ list,
                                                            const int* __restrict__ n_live,
                                                            float* __restrict__ embeds, int L) {
  extern __shared__ float4 px4[];  // [dp][2] float4 = [dp][8] floats
  float* px = (float*)px4;
  const int gw = W / patch, dp = 3 * patch * patch;
  const int b = blockIdx.z, g0 = blockIdx.y * EMB_PB, n = blockIdx.x * 256 + threadIdx.x;
  const int nl = n_live[b];
  if (g0 >= nl) return;
  const int* mine = list + (size_t)b * 4096 + g0;
  const int cnt = min(EMB_PB, nl - g0);
  const int prow = 3 * patch;  // bytes of one pixel row of a patch
  const int dpp = (dp + EMB_CH - 1) / EMB_CH * EMB_CH;  // rows of k past dp hold zeros
  for (int e = threadIdx.x; e < dpp * EMB_PB; e += 256) {
    const int j = e / dpp, k = e - j * dpp;  // consecutive threads: consecutive bytes of a patch row
    float v = 0.f;
    if (j < cnt && k < dp) {
      const int i = mine[j], r = i / gw, c = i - r * gw, y = k / prow, x = k - y * prow;
      v = (float)frame[(((size_t)b * H + (size_t)r * patch + y) * W + (size_t)c * patch) * 3 + x] / 127.5f - 1.0f;
    }
    px[k * EMB_PB + j] = v;
  }
  __syncthreads();
  if (n >= d) return;
  float acc[EMB_PB];
#pragma unroll
  for (int j = 0; j < EMB_PB; ++j) acc[j] = 0.f;
  // weights of EMB_CH values of k at a time, the next batch in flight behind the FMAs
  // (past the end the last row is fetched again and meets the zeros in LDS)
  uint16_t wa[EMB_CH], wb[EMB_CH];
  const bf16_t* wcol = w_proj + n;
#pragma unroll
  for (int u = 0; u < EMB_CH; ++u) wa[u] = wcol[(size_t)min(u, dp - 1) * d];
  for (int k0 = 0; k0 < dpp; k0 += EMB_CH) {
#pragma unroll
    for (int u = 0; u < EMB_CH; ++u) wb[u] = wcol[(size_t)min(k0 + EMB_CH + u, dp - 1) * d];
#pragma unroll
    for (int u = 0; u < EMB_CH; ++u) {
      const float w = __uint_as_float((uint32_t)wa[u] << 16);  // bf16 -> fp32
      const float4 a = px4[2 * (k0 + u)], c = px4[2 * (k0 + u) + 1];
      acc[0] = fmaf(a.x, w, acc[0]); acc[1] = fmaf(a.y, w, acc[1]);
      acc[2] = fmaf(a.z, w, acc[2]); acc[3] = fmaf(a.w, w, acc[3]);
      acc[4] = fmaf(c.x, w, acc[4]); acc[5] = fmaf(c.y, w, acc[5]);
      acc[6] = fmaf(c.z, w, acc[6]); acc[7] = fmaf(c.w, w, acc[7]);
    }
#pragma unroll
    for (int u = 0; u < EMB_CH; ++u) wa[u] = wb[u];
  }
#pragma unroll
  for (int j = 0; j < EMB_PB; ++j)
    if (j < cnt) embeds[((size_t)b * L + mine[j]) * d + n] = acc[j];
}

void launch_embed_patches(vlac_ctx* c, const uint8_t* frame, int B, int H, int W, int patch,
                          const bf16_t* w_proj, const int32_t* reuse_order, const int32_t* reuse_count,
                          int stride, const int32_t* layer_count, float* embeds, int L, hipStream_t st) {
  const int L_v = (H / patch) * (W / patch), d = c->cfg.d_model, dp = 3 * patch * patch;
  hipLaunchKernelGGL(embed_mark_kernel, dim3(B), dim3(256), 0, st, reuse_order, reuse_count, stride,
                     layer_count, c->cfg.n_layers, L_v, c->flags, c->embed_list, c->embed_n);
  hipLaunchKernelGGL(embed_patches_kernel, dim3((d + 255) / 256, (L_v + EMB_PB - 1) / EMB_PB, B), dim3(256),
                     (size_t)EMB_PB * ((dp + EMB_CH - 1) / EMB_CH * EMB_CH) * sizeof(float), st, frame, H, W,
                     patch, w_proj, d, c->embed_list,
                     c->embed_n, embeds, L);
}
