// Recomputed-row GEMMs of the sparse prefill and of the decode passes
// (Alg. 2 of VLA-Cache: K, V, and with them Q, O and the feed-forward, are
// computed for the rows outside P_reuse only; Sec. 3.1 for the projections).
//
// y[rows, N] = x[rows, K] . W[N, K]^T with few rows (tens to a few hundred)
// against large bf16 weights: the weights are the traffic, so the kernel is
// built to stream them from HBM exactly once at full rate.
//
//  * Weights and activations are both stored in fragment order (common.h), so
//    every operand fetch is one coalesced 16-byte load per lane and feeds a
//    v_mfma_f32_32x32x16_bf16 without any shuffling.
//  * The matrix-core A operand is the WEIGHT tile (32 output features x 16 k),
//    the B operand the activation tile (16 k x 32 rows); a lane of the result
//    holds one row and 4 x 4 consecutive features, which is what the fused
//    epilogues want (rotary partners, gate/up pairs and packed 8-byte stores in
//    one lane).
//  * A workgroup is 4 waves = 4 x 32 output features over all rows of its row
//    block (MT tiles of 32 rows, accumulators in registers).  Weight tiles go
//    global -> registers (each is used by exactly one wave, LDS would add
//    nothing); the activation tiles, shared by the 4 waves, are staged through
//    LDS, double buffered, 64 k per step.
//  * Few rows mean few output tiles, so K is split over S workgroups per tile to
//    fill 256 CUs; partial sums go to a workspace and the LAST workgroup to
//    arrive (atomic counter, no waiting) adds them in fixed order and runs the
//    epilogue: deterministic, no extra launch.
//  * Row counts live in device memory (they depend on the selection), the grid
//    is sized for the worst case and surplus workgroups leave at once.
//  * Workgroup ids are dealt round-robin to the 8 XCDs; row blocks of one weight
//    tile are mapped to the same XCD so that they share its L2.
#include "common.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const uint4* wp;    // weights, fragment order, 64 uint4 per tile
  const uint4* xp;    // activations, fragment order
  int NB;             // weight row blocks (32 output features each)
  int KS;             // K steps (64 k = 4 tiles each)
  const int* n_rows;  // device: rows in use
  int S, MB, P;       // split-K factor, row blocks, weight tiles * S
  float* partial;
  int* counters;
  GemmEpi e;
};

__device__ inline float silu_f(float x) { return x / (1.f + __expf(-x)); }

template <int EPI>
__device__ inline void epilogue_tile(const GemmEpi& e, int nb, int slot, int id, int g,
                                     const f32x16& acc) {
  const int b = id >> 16, pos = id & 0xffff;
  if constexpr (EPI == EPI_QKV) {
    const int hd = e.head_dim, bph = hd >> 5;
    const int nbq = e.n_q_heads * bph, nbk = e.n_kv_heads * bph;
    const size_t head_elems = (size_t)e.max_seq * hd;
    bf16_t* kvl = e.kv + (size_t)b * e.kv_stream_stride + e.kv_layer_off;
    if (nb < nbq + nbk) {
      // query or key block: rows 0..15 hold features f, rows 16..31 their rotary partners f + hd/2
      const bool isq = nb < nbq;
      const int nbl = isq ? nb : nb - nbq, head = nbl / bph, sb = nbl % bph;
      bf16_t* dst;
      int row;  // row of the fragment-ordered destination
      if (isq) {
        dst = e.qbuf + ((size_t)(slot >> 5) * e.n_q_heads + head) * (size_t)(hd >> 4) * 512;
        row = slot & 31;
      } else {
        dst = kvl + (size_t)head * head_elems + (size_t)(pos >> 5) * (hd >> 4) * 512;
        row = pos & 31;
      }
#pragma unroll
      for (int q4 = 0; q4 < 2; ++q4) {
        const int f1 = 16 * sb + 8 * q4 + 4 * g;
        const float4 c4 = *(const float4*)(e.rope_cos + (size_t)pos * (hd >> 1) + f1);
        const float4 s4 = *(const float4*)(e.rope_sin + (size_t)pos * (hd >> 1) + f1);
        const float cs[4] = {c4.x, c4.y, c4.z, c4.w}, sn[4] = {s4.x, s4.y, s4.z, s4.w};
        float o1[4], o2[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float x1 = acc[4 * q4 + k], x2 = acc[4 * (q4 + 2) + k];
          o1[k] = x1 * cs[k] - x2 * sn[k];
          o2[k] = x2 * cs[k] + x1 * sn[k];
        }
        const int f2 = f1 + (hd >> 1);
        *(uint2*)(dst + (size_t)(f1 >> 4) * 512 + ((row + (((f1 >> 3) & 1) << 5)) << 3) + (f1 & 7)) =
            make_uint2(pack_bf16x2(o1[0], o1[1]), pack_bf16x2(o1[2], o1[3]));
        *(uint2*)(dst + (size_t)(f2 >> 4) * 512 + ((row + (((f2 >> 3) & 1) << 5)) << 3) + (f2 & 7)) =
            make_uint2(pack_bf16x2(o2[0], o2[1]), pack_bf16x2(o2[2], o2[3]));
      }
    } else {
      // value block -> the cache's V tile: per 32 positions and 32 features, the
      // operand of the P.V product (key order inside a tile follows the score tile)
      const int nbl = nb - nbq - nbk, head = nbl / bph, ib = nbl % bph;
      const int pt = pos >> 5, pl = pos & 31, s = pl >> 4, r16 = pl & 15;
      const int gp = (r16 & 7) >> 2, ep = 4 * (r16 >> 3) + (r16 & 3);
      bf16_t* dst = kvl + (size_t)(e.n_kv_heads + head) * head_elems +
                    (((size_t)pt * bph + ib) * 2 + s) * 512 + (size_t)(32 * gp) * 8 + ep;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
        for (int k = 0; k < 4; ++k) dst[(8 * q4 + 4 * g + k) * 8] = f2bf(acc[4 * q4 + k]);
    }
  } else if constexpr (EPI == EPI_RESID) {
    const float* rs = e.resid_src + ((size_t)b * e.resid_seq_stride + pos) * e.d_model + nb * 32 + 4 * g;
    float* hp = e.h + ((size_t)b * e.max_seq + pos) * e.d_model + nb * 32 + 4 * g;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      float4 r = *(const float4*)(rs + 8 * q4);
      r.x += acc[4 * q4]; r.y += acc[4 * q4 + 1]; r.z += acc[4 * q4 + 2]; r.w += acc[4 * q4 + 3];
      *(float4*)(hp + 8 * q4) = r;
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    // rows 0..15 of the block: gate features, rows 16..31: the matching up features
#pragma unroll
    for (int q4 = 0; q4 < 2; ++q4) {
      const int ff = 16 * nb + 8 * q4 + 4 * g;
      float o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) o[k] = silu_f(acc[4 * q4 + k]) * acc[4 * (q4 + 2) + k];
      *(uint2*)(e.xf + frag_off(slot, ff, e.kc_f)) =
          make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
    }
  } else {  // EPI_LOGITS: slot is the stream
    float* out = e.logits + (size_t)slot * e.logits_stride + nb * 32 + 4 * g;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
      *(float4*)(out + 8 * q4) =
          make_float4(acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2], acc[4 * q4 + 3]);
  }
}

template <int MT, int EPI>
__global__ __launch_bounds__(256) void gemm_rows_kernel(GemmArgs a) {
  extern __shared__ uint4 lds[];  // [2][MT][256]: two stages of MT activation tiles x 4 k-tiles
  __shared__ int s_last;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // workgroup id -> (weight tile, split, row block); id % 8 is the XCD
  const int x = blockIdx.x, y = x >> 3;
  const int mb = y % a.MB, p = (y / a.MB) * 8 + (x & 7);
  if (p >= a.P) return;
  const int tile = p / a.S, s = p - tile * a.S;
  const int n_rows = *a.n_rows, row0 = mb * MT * 32;
  if (row0 >= n_rows) return;
  const int n_act = min(MT, (n_rows - row0 + 31) >> 5);
  const int nb = tile * 4 + w;
  const bool wave_on = nb < a.NB;
  const int KC = 4 * a.KS;
  const int q = a.KS / a.S, r = a.KS % a.S;
  const int ks0 = s * q + min(s, r), ks1 = ks0 + q + (s < r ? 1 : 0);
  const uint4* wsrc = a.wp + (size_t)(wave_on ? nb : a.NB - 1) * KC * 64 + lane;
  const uint4* xsrc = a.xp + (size_t)(row0 >> 5) * KC * 64 + tid;

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
  uint4 breg[3][4], areg[MT];

  auto load_b = [&](int ks, uint4(&dst)[4]) {
    const int k = min(ks, ks1 - 1);
#pragma unroll
    for (int c = 0; c < 4; ++c) dst[c] = wsrc[(size_t)(4 * k + c) * 64];
  };
  auto load_a = [&](int ks) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (mt < n_act) areg[mt] = xsrc[((size_t)mt * KC + 4 * ks) * 64];
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (mt < n_act) lds[(buf * MT + mt) * 256 + tid] = areg[mt];
  };
  auto step = [&](int ks, uint4(&bcur)[4]) {
    const int buf = (ks - ks0) & 1;
    __syncthreads();
    const bool more = ks + 1 < ks1;
    if (more) load_a(ks + 1);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bf16x8 bw = __builtin_bit_cast(bf16x8, bcur[c]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        if (mt < n_act) {
          const bf16x8 av = __builtin_bit_cast(bf16x8, lds[(buf * MT + mt) * 256 + c * 64 + lane]);
          acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw, av, acc[mt], 0, 0, 0);
        }
    }
    load_b(ks + 3, bcur);
    if (more) store_a(buf ^ 1);
  };

  load_a(ks0);
  load_b(ks0, breg[0]);
  load_b(ks0 + 1, breg[1]);
  load_b(ks0 + 2, breg[2]);
  store_a(0);
  for (int ks = ks0; ks < ks1; ks += 3) {
    step(ks, breg[0]);
    if (ks + 1 < ks1) step(ks + 1, breg[1]);
    if (ks + 2 < ks1) step(ks + 2, breg[2]);
  }

  if (a.S > 1) {
    // split-K: park the partial sums; the last workgroup of this (tile, row block) adds them up
    const size_t per_wave = (size_t)MT * 16 * 64;
    float* base = a.partial + ((size_t)(tile * a.MB + mb) * a.S) * 4 * per_wave;
    float* mine = base + ((size_t)s * 4 + w) * per_wave + lane;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (mt < n_act)
#pragma unroll
        for (int i = 0; i < 16; ++i) mine[(mt * 16 + i) * 64] = acc[mt][i];
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      int* cnt = a.counters + tile * a.MB + mb;
      const int old = atomicAdd(cnt, 1);
      s_last = (old == a.S - 1);
      if (old == a.S - 1) *cnt = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (mt < n_act)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float v = 0.f;
          for (int ss = 0; ss < a.S; ++ss)
            v += base[((size_t)ss * 4 + w) * per_wave + (mt * 16 + i) * 64 + lane];
          acc[mt][i] = v;
        }
  }

  if (!wave_on) return;
  const int g = lane >> 5;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    if (mt < n_act) {
      const int slot = row0 + mt * 32 + (lane & 31);
      if (slot < n_rows) {
        const int id = (EPI == EPI_LOGITS) ? 0 : a.e.rows[slot];
        epilogue_tile<EPI>(a.e, nb, slot, id, g, acc[mt]);
      }
    }
}

template <int MT, int EPI>
static hipError_t set_attr() {
  return hipFuncSetAttribute((const void*)gemm_rows_kernel<MT, EPI>,
                             hipFuncAttributeMaxDynamicSharedMemorySize, 2 * MT * 4096);
}

int gemm_init() {
  hipError_t e;
#define VLAC_SET(MT)                                                    \
  if ((e = set_attr<MT, EPI_QKV>()) != hipSuccess) return (int)e;       \
  if ((e = set_attr<MT, EPI_RESID>()) != hipSuccess) return (int)e;     \
  if ((e = set_attr<MT, EPI_SWIGLU>()) != hipSuccess) return (int)e;    \
  if ((e = set_attr<MT, EPI_LOGITS>()) != hipSuccess) return (int)e;
  VLAC_SET(1) VLAC_SET(4) VLAC_SET(9)
#undef VLAC_SET
  return 0;
}

template <int MT>
static void launch_mt(int epi, const GemmArgs& a, int grid, hipStream_t st) {
  const size_t shm = (size_t)2 * MT * 4096;
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_QKV>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_RESID:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_RESID>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_SWIGLU>), dim3(grid), dim3(256), shm, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_LOGITS>), dim3(grid), dim3(256), shm, st, a);
      break;
  }
}

void launch_gemm(vlac_ctx* c, int epi, const bf16_t* wp, int n_blocks, int kpad, const bf16_t* xp,
                 const int* n_rows, int rows_cap, const GemmEpi& e, hipStream_t st) {
  GemmArgs a;
  a.wp = (const uint4*)wp;
  a.xp = (const uint4*)xp;
  a.NB = n_blocks;
  a.KS = kpad / 64;
  a.n_rows = n_rows;
  a.partial = c->partial;
  a.counters = c->counters;
  a.e = e;
  const int MT = rows_cap <= 32 ? 1 : (rows_cap <= 128 ? 4 : 9);
  const int tiles = (n_blocks + 3) / 4;
  a.MB = (rows_cap + MT * 32 - 1) / (MT * 32);
  // split K until about two workgroups per CU exist
  int S = (512 + tiles * a.MB - 1) / (tiles * a.MB);
  if (S > a.KS) S = a.KS;
  if (S > 16) S = 16;
  while (S > 1 && (size_t)tiles * a.MB * S * 4 * MT * 16 * 64 > c->partial_floats) --S;
  if (tiles * a.MB > c->n_counters) S = 1;
  if (S < 1) S = 1;
  a.S = S;
  a.P = tiles * S;
  const int grid = ((a.P + 7) / 8) * 8 * a.MB;
  if (MT == 1) launch_mt<1>(epi, a, grid, st);
  else if (MT == 4) launch_mt<4>(epi, a, grid, st);
  else launch_mt<9>(epi, a, grid, st);
}
