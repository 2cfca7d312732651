// Token selection (Alg. 1 of VLA-Cache) and the layer-adaptive ratio (Sec. 3.4).
//
//   patch_terms_kernel   Eq. (sim): per patch the exact integers dot, |P_t|^2, |P_{t-1}|^2
//   select_rank_kernel   threshold (Sim >= tau, cross-multiplied in 128-bit integers),
//                        Top-k by exact rational comparison (Eq. topk), task-relevance
//                        quantile filter (Eq. ptask, Eq. pfinal)
//   select_compact_kernel  ascending index list and reuse order
//   layer_ratio_kernel   entropy ratio and Eq. (reuse_ratio), in fp64
//
// All of this is HBM/latency-bound integer work: 2*H*W*3 bytes of pixels per
// stream are read exactly once, with 16-byte loads over the contiguous run of
// image rows that one row of patches covers.
#include <mutex>

#include "common.h"

typedef unsigned __int128 u128;

// ---------------------------------------------------------------------------
// Eq. (sim) terms.  One workgroup per (patch row, stream).
// ---------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(256) void patch_terms_kernel(const uint8_t* __restrict__ prev,
                                                          const uint8_t* __restrict__ cur, int H,
                                                          int W, int patch,
                                                          uint32_t* __restrict__ terms) {
  extern __shared__ uint32_t acc[];  // [gw][3]
  const int gw = W / patch, gh = H / patch;
  const int b = blockIdx.y, pr = blockIdx.x, tid = threadIdx.x;
  const size_t base = ((size_t)b * H + (size_t)pr * patch) * W * 3;
  const int rowbytes = W * 3, pbytes = patch * 3, nbytes = patch * rowbytes;
  for (int i = tid; i < gw * 3; i += 256) acc[i] = 0;
  __syncthreads();
  for (int o = tid * VEC; o < nbytes; o += 256 * VEC) {
    uint32_t av[4] = {0, 0, 0, 0}, bv[4] = {0, 0, 0, 0};
    if constexpr (VEC == 16) {
      const uint4 a4 = *(const uint4*)(cur + base + o);
      const uint4 b4 = *(const uint4*)(prev + base + o);
      av[0] = a4.x; av[1] = a4.y; av[2] = a4.z; av[3] = a4.w;
      bv[0] = b4.x; bv[1] = b4.y; bv[2] = b4.z; bv[3] = b4.w;
    } else {
      av[0] = cur[base + o];
      bv[0] = prev[base + o];
    }
    const int c = o % rowbytes;
    int j = c / pbytes, within = c % pbytes;
    uint32_t d = 0, na = 0, nb = 0;
    auto flush = [&]() {
      if (d | na | nb) {
        atomicAdd(&acc[j * 3 + 0], d);
        atomicAdd(&acc[j * 3 + 1], na);
        atomicAdd(&acc[j * 3 + 2], nb);
      }
      d = na = nb = 0;
    };
    auto advance = [&](int n) {
      within += n;
      if (within == pbytes) {
        flush();
        within = 0;
        if (++j == gw) j = 0;
      }
    };
    if constexpr (VEC == 16) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (within + 4 <= pbytes) {  // the whole dword lies in one patch
          d = __builtin_amdgcn_udot4(av[k], bv[k], d, false);
          na = __builtin_amdgcn_udot4(av[k], av[k], na, false);
          nb = __builtin_amdgcn_udot4(bv[k], bv[k], nb, false);
          advance(4);
        } else {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t x = (av[k] >> (8 * q)) & 255u, y = (bv[k] >> (8 * q)) & 255u;
            d += x * y; na += x * x; nb += y * y;
            advance(1);
          }
        }
      }
    } else {
      d = av[0] * bv[0]; na = av[0] * av[0]; nb = bv[0] * bv[0];
      advance(1);
    }
    flush();
  }
  __syncthreads();
  const int Lv = gw * gh;
  for (int i = tid; i < gw * 3; i += 256)
    terms[((size_t)b * Lv + (size_t)pr * gw) * 3 + i] = acc[i];
}

void launch_patch_terms(const uint8_t* prev, const uint8_t* cur, int B, int H, int W, int patch,
                        uint32_t* terms, hipStream_t st) {
  const int gw = W / patch, gh = H / patch;
  const size_t shm = (size_t)gw * 3 * sizeof(uint32_t);
  const bool vec = ((size_t)patch * W * 3) % 16 == 0 && ((size_t)H * W * 3) % 16 == 0 &&
                   ((uintptr_t)prev % 16 == 0) && ((uintptr_t)cur % 16 == 0);
  dim3 grid(gh, B);
  if (vec)
    hipLaunchKernelGGL(patch_terms_kernel<16>, grid, dim3(256), shm, st, prev, cur, H, W, patch, terms);
  else
    hipLaunchKernelGGL(patch_terms_kernel<1>, grid, dim3(256), shm, st, prev, cur, H, W, patch, terms);
}

// ---------------------------------------------------------------------------
// Threshold, Top-k, relevance filter.
// ---------------------------------------------------------------------------
struct Frac { uint64_t num, den; };  // Sim^2 as an exact fraction

__device__ inline Frac sim_fraction(uint32_t dot, uint32_t na, uint32_t nb) {
  // two all-zero patches are identical, exactly one all-zero patch is dissimilar
  if (na == 0 && nb == 0) return {1, 1};
  if (na == 0 || nb == 0) return {0, 1};
  return {(uint64_t)dot * dot, (uint64_t)na * nb};
}

#define SEL_MAX_LV 4096
struct LayerMask { uint32_t w[16]; };  // bit l set = layer l is averaged over (<= 512 layers)

// grid (ceil(L_v / 16), B).  flags[b, i] = 1 iff patch i is in P_final.
// A workgroup ranks 256 / SEL_LPT patches, SEL_LPT lanes to a patch: every lane counts, over
// its share of the other patches, those that come before its patch (by similarity for Top-k,
// by score for the relevance quantile), and the counts are added up across the lanes
// (integers: the result does not depend on how the patches are dealt).  Every workgroup
// first builds the stream's similarities and scores in LDS, so many lanes per patch pay
// while the launch is small (16 lanes: 8 us instead of 46 us at one stream of 256 patches)
// and one lane per patch is right once the streams alone fill the chip.
template <int SEL_LPT>
__global__ __launch_bounds__(256) void select_rank_kernel(
    const uint32_t* __restrict__ terms, int L_v, uint64_t tn2, uint64_t td2, int top_k,
    const float* __restrict__ attn_mean, int n_layers, int B, LayerMask layer_mask, int n_rel, uint8_t* __restrict__ flags, float* __restrict__ relevance) {
  __shared__ double approx[SEL_MAX_LV];
  __shared__ float score[SEL_MAX_LV];
  __shared__ uint8_t pass[SEL_MAX_LV];
  const int b = blockIdx.y, tid = threadIdx.x;
  const uint32_t* t = terms + (size_t)b * L_v * 3;
  for (int j = tid; j < L_v; j += 256) {
    const Frac f = sim_fraction(t[j * 3], t[j * 3 + 1], t[j * 3 + 2]);
    pass[j] = (u128)f.num * td2 >= (u128)tn2 * f.den;
    approx[j] = (double)f.num / (double)f.den;
    float s = 0.f;
    if (attn_mean) {
      int n = 0;
      for (int l = 0; l < n_layers; ++l)
        if ((layer_mask.w[l >> 5] >> (l & 31)) & 1u) {
          s += attn_mean[((size_t)l * B + b) * L_v + j];
          ++n;
        }
      s = s / (float)(n > 0 ? n : 1);
    }
    score[j] = s;
  }
  __syncthreads();
  constexpr int SEL_PPW = 256 / SEL_LPT;
  const int sub = tid % SEL_LPT;
  const int i = blockIdx.x * SEL_PPW + tid / SEL_LPT;
  const bool live = i < L_v;           // (a patch's 16 lanes lie in one wave and leave together)
  const int ii = live ? i : 0;
  const bool passed = pass[ii] && top_k > 0;
  int rank = 0, rr = 0;
  if (passed) {
    // rank among the passers: higher similarity first, ties -> lower index
    const double ai = approx[ii];
    const Frac fi = sim_fraction(t[ii * 3], t[ii * 3 + 1], t[ii * 3 + 2]);
    for (int j = sub; j < L_v; j += SEL_LPT) {
      if (!pass[j] || j == ii) continue;
      const double dlt = approx[j] - ai;
      bool beats;
      if (dlt > 1e-12) beats = true;
      else if (dlt < -1e-12) beats = false;
      else {  // too close for fp64: exact cross-multiplication
        const Frac fj = sim_fraction(t[j * 3], t[j * 3 + 1], t[j * 3 + 2]);
        const u128 lhs = (u128)fj.num * fi.den, rhs = (u128)fi.num * fj.den;
        beats = lhs > rhs || (lhs == rhs && j < ii);
      }
      rank += beats;
    }
  }
  const float si = score[ii];
  if (attn_mean && n_rel > 0) {
    // rank by score descending, ties -> lower index
    for (int j = sub; j < L_v; j += SEL_LPT) rr += (score[j] > si) || (score[j] == si && j < ii);
  }
#pragma unroll
  for (int o = SEL_LPT / 2; o > 0; o >>= 1) {
    rank += __shfl_xor(rank, o);
    rr += __shfl_xor(rr, o);
  }
  if (!live || sub != 0) return;
  bool keep = passed && rank < top_k;
  if (attn_mean) {
    if (keep && n_rel > 0) keep = rr >= n_rel;
    relevance[(size_t)b * L_v + i] = si;
  } else {
    relevance[(size_t)b * L_v + i] = 0.f;
  }
  flags[(size_t)b * L_v + i] = keep;
}

// grid (B).  Ascending list, count, and the list ordered by (score asc, index asc).
// The kept tokens are compacted first (ascending index, with their scores, in LDS); the
// place of a kept token in the reuse order is then the number of kept tokens that come
// before it, counted over the compact list only: its k-th entry precedes the i-th if its
// score is lower, or equal with k < i (the compact list ascends by index).
__global__ __launch_bounds__(256) void select_compact_kernel(
    const uint8_t* __restrict__ flags, const float* __restrict__ relevance, int L_v,
    int32_t* __restrict__ out_idx, int32_t* __restrict__ out_order, int32_t* __restrict__ out_count,
    float* __restrict__ out_relevance, int stride) {
  __shared__ float cscore[SEL_MAX_LV];
  __shared__ int cidx[SEL_MAX_LV];
  __shared__ int wsum[4];
  __shared__ int base_s;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) base_s = 0;
  __syncthreads();
  for (int c0 = 0; c0 < L_v; c0 += 256) {
    const int i = c0 + tid;
    int f = 0;
    float sc = 0.f;
    if (i < L_v) {
      f = flags[(size_t)b * L_v + i];
      sc = relevance[(size_t)b * L_v + i];
      if (out_relevance) out_relevance[(size_t)b * L_v + i] = sc;
    }
    const unsigned long long bal = __ballot(f);
    const int inwave = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) wsum[w] = __popcll(bal);
    __syncthreads();
    int off = base_s;
    for (int k = 0; k < w; ++k) off += wsum[k];
    if (f) {
      const int k = off + inwave;
      cidx[k] = i;
      cscore[k] = sc;
      if (k < stride) out_idx[(size_t)b * stride + k] = i;
    }
    __syncthreads();
    if (tid == 0) base_s += wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
  const int n = base_s;
  if (tid == 0) out_count[b] = n;
  for (int i = tid; i < n; i += 256) {
    const float si = cscore[i];
    int ord = 0;
    for (int k = 0; k < n; ++k) {
      const float sk = cscore[k];
      ord += (sk < si) || (sk == si && k < i);
    }
    if (ord < stride) out_order[(size_t)b * stride + ord] = cidx[i];
  }
}

void launch_select(const uint32_t* terms, int B, int L_v, int tau_num, int tau_den, int top_k,
                   const float* attn_mean, int n_layers, const uint8_t* layer_mask_host, int n_rel,
                   uint8_t* flags, float* relevance_ws, int32_t* out_idx, int32_t* out_order,
                   int32_t* out_count, float* out_relevance, int stride, hipStream_t st) {
  const uint64_t tn2 = (uint64_t)tau_num * (uint64_t)tau_num;
  const uint64_t td2 = (uint64_t)tau_den * (uint64_t)tau_den;
  LayerMask lm;
  for (int i = 0; i < 16; ++i) lm.w[i] = 0;
  for (int l = 0; l < n_layers && l < 512; ++l)
    if (!layer_mask_host || layer_mask_host[l]) lm.w[l >> 5] |= 1u << (l & 31);
  const long long patches = (long long)B * L_v;
#define VLAC_RANK(LPT_)                                                                            \
  hipLaunchKernelGGL(select_rank_kernel<LPT_>, dim3((L_v * LPT_ + 255) / 256, B), dim3(256), 0, st, \
                     terms, L_v, tn2, td2, top_k, attn_mean, n_layers, B, lm, n_rel, flags, relevance_ws)
  if (patches <= 16384) VLAC_RANK(16);
  else if (patches <= 65536) VLAC_RANK(4);
  else VLAC_RANK(1);
#undef VLAC_RANK
  hipLaunchKernelGGL(select_compact_kernel, dim3(B), dim3(256), 0, st, flags, relevance_ws, L_v,
                     out_idx, out_order, out_count, out_relevance, stride);
}

// ---------------------------------------------------------------------------
// Sec. 3.4.  grid (B), fp64 throughout; sums are fixed-shape trees, so the
// result does not depend on scheduling.
// ---------------------------------------------------------------------------
#define RATIO_MAX_LAYERS 512

__global__ __launch_bounds__(1024) void layer_ratio_kernel(
    const float* __restrict__ attn_mean, int n_layers, int B, int L_v, float gain_k,
    const int32_t* __restrict__ reuse_count, float* __restrict__ out_alpha,
    int32_t* __restrict__ out_layer_count) {
  __shared__ double ent[RATIO_MAX_LAYERS];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // a wave per layer (layers w, w + 16, ...): its sums are shuffle trees of fixed shape
  for (int l = w; l < n_layers; l += 16) {
    const float* a = attn_mean + ((size_t)l * B + b) * L_v;
    double s = 0;
    for (int v = lane; v < L_v; v += 64) s += (double)a[v];
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    const double tot = s;
    double e = 0;
    if (tot > 0)
      for (int v = lane; v < L_v; v += 64) {
        const double p = (double)a[v] / tot;
        if (p > 0) e -= p * log(p);
      }
    for (int o = 32; o > 0; o >>= 1) e += __shfl_xor(e, o);
    if (lane == 0) ent[l] = tot > 0 ? e : 0.0;
  }
  __syncthreads();
  if (tid == 0) {
    double cum = 0, best = 0;
    const int cnt = reuse_count ? reuse_count[b] : 0;
    for (int l = 0; l < n_layers; ++l) {
      if (l > 0 && ent[l - 1] > 0) cum += (ent[l - 1] - ent[l]) / ent[l - 1];
      double al = (double)gain_k * cum;
      al = al < 0 ? 0 : (al > 1 ? 1 : al);
      best = al > best ? al : best;
      const float af = (float)best;
      out_alpha[(size_t)b * n_layers + l] = af;
      if (out_layer_count)
        out_layer_count[(size_t)b * n_layers + l] = (int)floorf(af * (float)(cnt > 0 ? cnt : 0));
    }
  }
}

void launch_layer_ratio(const float* attn_mean, int n_layers, int B, int L_v, float gain_k,
                        const int32_t* reuse_count, float* out_alpha, int32_t* out_layer_count,
                        hipStream_t st) {
  hipLaunchKernelGGL(layer_ratio_kernel, dim3(B), dim3(1024), 0, st, attn_mean, n_layers, B, L_v,
                     gain_k, reuse_count, out_alpha, out_layer_count);
}

// ---------------------------------------------------------------------------
// Alg. 1 for callers that cannot allocate: the same three kernels, with their scratch (the
// patch terms, the score of every patch and the selection flags, which vlac_select_static
// keeps in its context) in a fixed array in device memory.  Every GPU holds its own copy of
// the array at its own address; host code only ever uses the address that
// hipGetSymbolAddress returns for the current device, never the array's name.  Nothing in
// the array has to start at zero: patch_terms_kernel writes all terms of the call's patches,
// select_rank_kernel all their scores and flags, before anything reads them.
// ---------------------------------------------------------------------------
namespace {

constexpr size_t kNoAllocPatches = VLAC_NOALLOC_MAX_PATCHES;
constexpr size_t kTermsOff = 0;                                   // uint32 [patches][3]
constexpr size_t kScoreOff = kTermsOff + kNoAllocPatches * 12;    // float  [patches]
constexpr size_t kFlagsOff = kScoreOff + kNoAllocPatches * 4;     // uint8  [patches]
constexpr size_t kScratchBytes = kFlagsOff + kNoAllocPatches;

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // per device: where that GPU holds `scratch`

// The address of the current device's copy of the array (looked up once per device).
hipError_t scratch_of_current_device(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (unsigned char*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

int select_scratch_init() {
  unsigned char* p = nullptr;
  return (int)scratch_of_current_device(&p);
}

extern "C" int vlac_select_static_noalloc(const uint8_t* frame_prev, const uint8_t* frame_cur, int B, int H,
                                          int W, int patch, int tau_num, int tau_den, int top_k,
                                          const float* attn_mean, int n_layers, const uint8_t* layer_mask,
                                          float tau_task, int32_t* out_idx, int32_t* out_order,
                                          int32_t* out_count, float* out_relevance, int stride,
                                          void* stream) {
  if (!frame_prev || !frame_cur || !out_idx || !out_order || !out_count) return VLAC_E_NULL;
  if (B < 1 || B > 32767) return VLAC_E_RANGE;
  if (patch < 1 || patch > 64 || H < 1 || W < 1) return VLAC_E_RANGE;
  if (H % patch || W % patch) return VLAC_E_SHAPE;
  const long L_v = (long)(H / patch) * (W / patch);
  if (L_v > SEL_MAX_LV) return VLAC_E_RANGE;
  if ((size_t)B * (size_t)L_v > kNoAllocPatches) return VLAC_E_RANGE;  // beyond the fixed scratch
  if (tau_den < 1 || tau_num < 0 || tau_num > tau_den) return VLAC_E_RANGE;
  if (top_k < 0 || top_k > L_v) return VLAC_E_RANGE;
  if (stride < top_k || stride < 1) return VLAC_E_SHAPE;
  if (tau_task != tau_task) return VLAC_E_RANGE;  // NaN
  if (attn_mean && (n_layers < 1 || n_layers > 512)) return VLAC_E_RANGE;
  int n_rel = 0;
  if (attn_mean) {
    // the L_v - floor(tau_task * L_v) highest-scoring tokens are task-relevant
    const double keep = floor((double)tau_task * (double)L_v);
    const double nr = (double)L_v - keep;
    n_rel = nr < 0 ? 0 : (nr > (double)L_v ? (int)L_v : (int)nr);
  }
  unsigned char* ws = nullptr;
  if (scratch_of_current_device(&ws) != hipSuccess) {
    (void)hipGetLastError();
    return VLAC_E_HIP;
  }
  uint32_t* terms = (uint32_t*)(ws + kTermsOff);
  float* score = (float*)(ws + kScoreOff);
  uint8_t* flags = (uint8_t*)(ws + kFlagsOff);
  hipStream_t st = (hipStream_t)stream;
  launch_patch_terms(frame_prev, frame_cur, B, H, W, patch, terms, st);
  launch_select(terms, B, (int)L_v, tau_num, tau_den, top_k, attn_mean, attn_mean ? n_layers : 0, layer_mask,
                n_rel, flags, score, out_idx, out_order, out_count, out_relevance, stride, st);
  return hipGetLastError() == hipSuccess ? VLAC_OK : VLAC_E_HIP;
}
