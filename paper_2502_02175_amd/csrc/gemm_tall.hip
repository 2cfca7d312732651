// Recomputed-row GEMMs with MANY rows (batched streams: thousands of rows per layer;
// Alg. 2 of VLA-Cache over the rows outside P_reuse of every stream at once).
//
// With thousands of rows the weights are no longer the traffic: the GEMM is bound by the
// matrix cores, and behind them by what the L2 delivers to a CU (measured here: about 20
// bytes per clock and CU, whatever the access pattern), so the operand bytes fetched per
// MFMA and the number of other instructions per MFMA are what has to be kept small.
//
//  * A workgroup is 8 waves (two per SIMD, so that one computes while the other waits);
//    a wave owns 2 blocks of 32 output features over all 4 row tiles of its row block:
//    8 accumulator tiles, and one k-tile is 8 MFMAs for 2 weight tiles + 4 activation
//    tiles fetched.  The workgroup tile is 512 features x 128 rows.
//  * Operands are in fragment order (common.h).  Weight tiles go global -> registers (no
//    other wave wants them): a ring of 6 k-tiles, the slot of a k-tile is refilled with
//    the tile 6 ahead as soon as its MFMAs are issued, so that loads are spread over the
//    step and have a step and a half of matrix work to land (L2 latency: the row blocks
//    of one weight tile run side by side on one XCD, all but one of them hit its L2).
//  * Activation tiles are shared by the 8 waves through LDS, 64 k per step, and are
//    copied global -> LDS directly (global_load_lds_dwordx4: lane l's 16 bytes land at
//    base + 16 l, which is the fragment order itself), two steps ahead, into a ring of 3
//    buffers: no staging registers, no LDS store instructions, one barrier per step.
//  * K is split only where tiles x row blocks leave half the chip idle, and only in the
//    residual GEMMs (O, FFN-down), whose consumer (residual add + RMSNorm) can add the
//    partial rows up: the split factor follows from the row count on the device
//    (tall_resid_splits).  Everywhere else tiles x row blocks fill the chip by themselves.
//  * Tried and measured, not kept: 4 waves x 4 feature blocks (one wave per SIMD: 12%
//    slower), staging the activation tiles through registers (the extra registers and
//    LDS stores cost 3%), a 256 x 256 tile whose weight tiles are fetched by two waves
//    each (the second fetch hits L1, but the kernel is 5% slower), a persistent grid that
//    deals the work items of the actual row count round-robin (2% slower than letting
//    the hardware dispatch one workgroup per item), a weight ring of 8 k-tiles instead of
//    6 (no faster: the loop does not wait for latency), a raised wave priority around
//    the MFMAs of a k-tile (+-1 %).  The same 8-wave design with one
//    feature block per wave, up to 8 row tiles and split K, tried for ONE stream's prefill
//    (33..1023 rows) in place of the 4-wave kernel of gemm.hip, was no faster at any row
//    count (109 rows: 6.0 vs 5.8 ms per prefill; 248 rows: 8.4 vs 8.2 ms).
#include "gemm_epi.h"

namespace {

constexpr int TALL_W = 8;   // waves per workgroup
constexpr int XBUF = 3;     // LDS buffers of 4 row tiles x 4 k-tiles

// (split s of S: this workgroup covers the 64-k steps [ks0, ks0 + KS) of the a.KS there are)
// NF: feature blocks per wave (2: the workgroup tile is 512 features wide, 1: 256)
template <int NF, int NA, int EPI, bool F16>
__device__ __forceinline__ void tall_body(const GemmArgs& a, uint4* lds, int tile, int mb, int n_rows,
                                          int s, int S) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int row0 = mb * 128;
  const int KC = 4 * a.KS;
  const int kq = a.KS / S, kr = a.KS % S;
  const int ks0 = s * kq + min(s, kr), KS = kq + (s < kr ? 1 : 0);
  const int nb0 = tile * (TALL_W * NF) + w * NF;
  const uint4* wsrc[NF];
#pragma unroll
  for (int fb = 0; fb < NF; ++fb)
    wsrc[fb] = a.wp + ((size_t)min(nb0 + fb, a.NB - 1) * KC + 4 * ks0) * 64 + lane;
  // this wave copies activation tiles j = 2 w, 2 w + 1 of a step's 16 (row tile j / 4, k-tile j % 4)
  const int mt0 = w >> 1, c0 = (w & 1) * 2;
  const uint4* xsrc = a.xp + ((size_t)((row0 >> 5) + mt0) * KC + 4 * ks0 + c0) * 64 + lane;
  uint4* xdst = lds + mt0 * 256 + c0 * 64;

  f32x16 acc[NF][NA];
#pragma unroll
  for (int fb = 0; fb < NF; ++fb)
#pragma unroll
    for (int mt = 0; mt < NA; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[fb][mt][i] = 0.f;

  uint4 W[6][NF];
  const int last_kt = 4 * KS - 1;
  auto load_w = [&](int kt, uint4(&dst)[NF]) {
    const size_t k = (size_t)min(kt, last_kt) * 64;
#pragma unroll
    for (int fb = 0; fb < NF; ++fb) dst[fb] = wsrc[fb][k];
  };
  // Activation tiles of step i -> LDS buffer i % 3 (row tiles past the block's last are
  // never read and not copied).  The copies are written as inline assembly on purpose:
  // the compiler treats its own LDS-direct loads as possibly aliasing every LDS read and
  // drains the whole load queue (the weight ring with it) before the next one.  So the
  // compiler does not know about these two loads per step, and the waits for them are
  // placed by hand (loads return in issue order, and nothing moves across the asm
  // statements, so the count of younger loads is fixed: see the step macro).  Its own
  // waits for the weight tiles can only come out longer than needed, never shorter.
  const uint32_t xdst0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)xdst);
  auto copy_x = [&](int i, int buf) {
    if (mt0 < NA) {
      const uint4* src = xsrc + (size_t)min(i, KS - 1) * 256;
      const uint32_t dst = xdst0 + buf * 16384;
      asm volatile(
          "s_mov_b32 m0, %0\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %1, off\n\t"
          "global_load_lds_dwordx4 %1, off offset:1024"  // next k-tile: + 1 KiB on both sides
          :
          : "s"(dst), "v"(src)
          : "memory", "m0");
    }
  };
  auto ktile = [&](int i, int c, int buf, uint4(&Ws)[NF]) {
    uint4 xf[NA];
#pragma unroll
    for (int mt = 0; mt < NA; ++mt) xf[mt] = lds[(buf * 4 + mt) * 256 + c * 64 + lane];
#pragma unroll
    for (int fb = 0; fb < NF; ++fb)
#pragma unroll
      for (int mt = 0; mt < NA; ++mt) acc[fb][mt] = mfma32<F16>(Ws[fb], xf[mt], acc[fb][mt]);
    load_w(4 * i + c + 6, Ws);
  };
  // Step i at phase ph = i % 3 of the unrolled loop: its k-tiles sit in slots
  // (4 ph + c) % 6 and its activation tiles in LDS buffer ph.  They were asked for at the
  // start of step i - 2; behind them this wave has issued 2 x 4 NF weight loads and the two
  // copies of step i + 1, so "at most 8 NF + 2 loads outstanding" means they have landed; the
  // barrier then makes that true for the copies of all 8 waves, and says that every wave
  // is done with step i - 1, whose buffer takes the tiles of step i + 2.
  // (In the one or two steps after the last full turn of the loop the count does not hold:
  // the weight loads of those steps refill slots that nobody reads any more, and the
  // compiler drops them.  There the wait is for everything.)
#define VLAC_TALL_STEP(i, ph, s0, s1, s2, s3, ALL)           \
  {                                                          \
    if (ALL) VLAC_VMCNT(0);                                  \
    else if (NF == 2) VLAC_VMCNT(18);                        \
    else VLAC_VMCNT(10);                                     \
    __syncthreads();                                         \
    copy_x((i) + 2, ((ph) + 2) % 3);                         \
    ktile((i), 0, ph, W[s0]);                                \
    ktile((i), 1, ph, W[s1]);                                \
    ktile((i), 2, ph, W[s2]);                                \
    ktile((i), 3, ph, W[s3]);                                \
  }

  copy_x(0, 0);
  copy_x(1, 1);
#pragma unroll
  for (int kt = 0; kt < 6; ++kt) load_w(kt, W[kt]);
  // both copies; the 6 NF weight loads fly on
  if (NF == 2) VLAC_VMCNT(12);
  else VLAC_VMCNT(6);
  int i = 0;
  for (; i + 3 <= KS; i += 3) {
    VLAC_TALL_STEP(i, 0, 0, 1, 2, 3, false)
    VLAC_TALL_STEP(i + 1, 1, 4, 5, 0, 1, false)
    VLAC_TALL_STEP(i + 2, 2, 2, 3, 4, 5, false)
  }
  if (i < KS) {
    VLAC_TALL_STEP(i, 0, 0, 1, 2, 3, true)
    if (i + 1 < KS) VLAC_TALL_STEP(i + 1, 1, 4, 5, 0, 1, true)
  }
#undef VLAC_TALL_STEP
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no copy outlives the loop

  const int g = lane >> 5;
  if (a.wscale) {  // weights expanded from e4m3 codes: the scale of every output feature
#pragma unroll
    for (int fb = 0; fb < NF; ++fb)
      if (nb0 + fb < a.NB) {
#pragma unroll
        for (int mt = 0; mt < NA; ++mt) scale_tile(a.wscale, nb0 + fb, g, acc[fb][mt]);
      }
  }
  if (EPI == EPI_RESID && S > 1) {
    // split K: the partial rows [split][row][feature] are left to the row kernel that follows
    // (residual add + RMSNorm), which adds the splits up in order
#pragma unroll
    for (int mt = 0; mt < NA; ++mt) {
      const int slot = row0 + mt * 32 + (lane & 31);
      if (slot < n_rows) {
#pragma unroll
        for (int fb = 0; fb < NF; ++fb)
          if (nb0 + fb < a.NB) {
            float* dst = a.e.rpart + ((size_t)s * a.e.rpart_rows + slot) * a.e.d_model + (nb0 + fb) * 32 + 4 * g;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
              *(float4*)(dst + 8 * q4) = make_float4(acc[fb][mt][4 * q4], acc[fb][mt][4 * q4 + 1],
                                                     acc[fb][mt][4 * q4 + 2], acc[fb][mt][4 * q4 + 3]);
          }
      }
    }
    return;
  }
#pragma unroll
  for (int mt = 0; mt < NA; ++mt) {
    const int slot = row0 + mt * 32 + (lane & 31);
    if (slot < n_rows) {
      const int id = (EPI == EPI_LOGITS) ? 0 : a.e.rows[slot];
#pragma unroll
      for (int fb = 0; fb < NF; ++fb)
        if (nb0 + fb < a.NB) epilogue_tile<EPI, F16>(a.e, nb0 + fb, slot, id, g, acc[fb][mt]);
    }
  }
}

template <int EPI, bool F16>
__global__ __launch_bounds__(512) void gemm_tall_kernel(GemmArgs a) {
  __shared__ uint4 lds[XBUF * 4 * 256];  // 3 stages of 4 activation tiles x 4 k-tiles
  // Work items are (weight tile, K split, row block) triples, listed with the row blocks of
  // one tile and split next to each other, and the list is cut into eight equal runs, one
  // per XCD (workgroup id % 8): an XCD's workgroups then share weight k-tiles through its
  // L2 as they start in id order, and every XCD gets the same number of items whatever the
  // tile count is.  The grid is sized for the largest possible row count and split factor;
  // the items of the actual row count come first in every XCD's run, and a workgroup that
  // finds none costs next to nothing (measured against a persistent grid that deals the
  // items round-robin, the hardware's dynamic dispatch wins).
  // (a.S > 1, residual epilogue only: how many K splits are used follows from the row
  // count, see tall_resid_splits)
  const int n_rows = a.n_rows_val >= 0 ? a.n_rows_val : *a.n_rows;
  if (n_rows < a.rows_lo) return;  // the one-stream kernel's share
  const int MBn = (n_rows + 127) >> 7;
  const TallPlan pl = tall_plan(a.NB, MBn, a.KS, EPI == EPI_RESID ? a.S : 1);
  const int S = pl.S;
  const int items = pl.tiles * S * MBn, per = (items + 7) >> 3;
  const int j = blockIdx.x >> 3, i = (blockIdx.x & 7) * per + j;
  if (j >= per || i >= items) return;
  const int vt = i / MBn, mb = i - vt * MBn;
  const int tile = vt / S, s = vt - tile * S;
  const int row0 = mb * 128;
  const int na = min(4, (n_rows - row0 + 31) >> 5);
  if (pl.nf == 2) {
    switch (na) {
      case 1: tall_body<2, 1, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      case 2: tall_body<2, 2, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      case 3: tall_body<2, 3, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      default: tall_body<2, 4, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
    }
  } else {
    switch (na) {
      case 1: tall_body<1, 1, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      case 2: tall_body<1, 2, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      case 3: tall_body<1, 3, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
      default: tall_body<1, 4, EPI, F16>(a, lds, tile, mb, n_rows, s, S); break;
    }
  }
}

template <bool F16>
void launch_tall(int epi, const GemmArgs& a, int grid, hipStream_t st) {
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_QKV, F16>), dim3(grid), dim3(512), 0, st, a);
      break;
    case EPI_RESID:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_RESID, F16>), dim3(grid), dim3(512), 0, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_SWIGLU, F16>), dim3(grid), dim3(512), 0, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_LOGITS, F16>), dim3(grid), dim3(512), 0, st, a);
      break;
  }
}

__global__ __launch_bounds__(256) void expand_e4m3_kernel(const uint4* __restrict__ codes,
                                                          uint4* __restrict__ tiles, size_t n) {
  // thread = one lane's slot: the 8 codes of k-tile 2c and the 8 of k-tile 2c + 1
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint4 slot = codes[i];
  const size_t pair = i >> 6, lane = i & 63;
  tiles[(2 * pair) * 64 + lane] = e4m3_slot_half(slot, 0);
  tiles[(2 * pair + 1) * 64 + lane] = e4m3_slot_half(slot, 1);
}

}  // namespace

void launch_expand_e4m3(const uint4* codes, uint4* tiles, size_t n_slots, hipStream_t st) {
  const size_t n = n_slots * 64;
  hipLaunchKernelGGL(expand_e4m3_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, codes, tiles, n);
}

void launch_gemm_tall(bool f16, int epi, GemmArgs& a, int rows_cap, int S_max, hipStream_t st) {
  a.S = (epi == EPI_RESID && S_max > 1) ? S_max : 1;
  a.MB = (rows_cap + 127) / 128;
  a.P = 0;
  // the grid covers the most work items any row count up to rows_cap can give: of both tile
  // widths and every split factor the plan can choose
  int most = 0;
  for (int mb = 1; mb <= a.MB; ++mb) {
    const TallPlan pl = tall_plan(a.NB, mb, a.KS, a.S);
    most = std::max(most, pl.tiles * pl.S * mb);
  }
  const int grid = ((most + 7) / 8) * 8;
  if (f16) launch_tall<true>(epi, a, grid, st);
  else launch_tall<false>(epi, a, grid, st);
}
