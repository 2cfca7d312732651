// Recomputed-row GEMMs with MANY rows, second kernel: both operands through LDS
// (Alg. 2 of VLA-Cache over the rows outside P_reuse of many streams at once; the QKV and
// gate/up projections, which complete their sums inside the kernel).
//
// The kernel of gemm_tall.hip keeps a 512-feature x 128-row tile per workgroup and fetches
// 20 KiB of operands per 64 MFMAs; what the L2 delivers to a CU bounds it.  Here a workgroup
// owns 256 features x 256 rows (16 KiB per 64 MFMAs), and both operand tiles are shared
// through LDS:
//
//  * 4 waves, one per SIMD; a wave owns 4 feature blocks x 4 row tiles = 16 accumulator
//    tiles (256 registers), and one k-tile is 16 MFMAs for 8 operand fragments read from LDS.
//  * Operands are in fragment order (common.h): a tile is 1 KiB that a wave copies global ->
//    LDS as it lies (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16 l) and
//    reads back with one 16-byte LDS read per lane, conflict-free.
//  * A stage is 32 k: 16 weight tiles + 16 activation tiles = 32 KiB; a ring of 5 stages
//    (all 160 KiB of a CU's LDS), copies run 4 stages ahead.  Every wave copies 8 tiles per stage, whatever the row
//    count (tiles past the end are clamped to a valid one and never read), so that the
//    number of copies in flight is the same for every wave at every step: the copies are
//    inline assembly that the compiler does not see, and their waits are placed by hand.
//  * One barrier per stage, placed between the MFMAs of its two k-tiles: the fragments of a
//    k-tile are read while the MFMAs of the one before run, across the barrier as well.
//  * Row blocks of 192 or 128 rows (a wave owns 4 x 3 or 4 x 2 tiles) where that takes fewer
//    rounds of 256 work items' worth than blocks of 256 (tall2_plan, evaluated on the device
//    from the row count).
#include "gemm_epi.h"

namespace {

#ifndef VLAC_T2_RING
#define VLAC_T2_RING 5
#endif
constexpr int T2_RING = VLAC_T2_RING;  // LDS stages: 5 x 32 KiB is all the LDS of a CU
// copies younger than the stage a step waits for: those of the T2_RING - 2 stages behind it
#if VLAC_T2_RING == 5
#define VLAC_T2_WAIT() VLAC_VMCNT(24)
#elif VLAC_T2_RING == 4
#define VLAC_T2_WAIT() VLAC_VMCNT(16)
#else
#error "add the wait for this ring size"
#endif
constexpr int T2_STAGE = 2048;        // uint4 per stage: 32 tiles of 64

// RT: row tiles per wave (4: blocks of 256 rows, 3: of 192, 2: of 128); NA: how many of them hold rows
template <int RT, int NA, int EPI, bool F16>
__device__ __forceinline__ void tall2_body(const GemmArgs& a, uint4* lds, int tile, int mb, int n_rows) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = w & 1, wj = w >> 1;  // feature half, row interleave
  const int KC = 4 * a.KS, n_steps = 2 * a.KS;
  const int row0 = mb * (64 * RT);
  const int nb0 = tile * 8;
  // This wave copies, per stage, the weight tiles of feature blocks 2w, 2w + 1 and the
  // activation tiles of row tiles 2w, 2w + 1 of the block (both k-tiles of each: 2 KiB that
  // lie together in global memory and in LDS).  Row blocks of 128 rows have 4 row tiles:
  // waves 2 and 3 copy tiles 4..7 all the same (clamped, unread).
  const uint4* src[4];
  uint32_t dst[4];
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int fb = 2 * w + p;
    src[p] = a.wp + ((size_t)min(nb0 + fb, a.NB - 1) * KC) * 64 + lane;
    dst[p] = lds0 + (uint32_t)(fb * 2) * 1024u;
    const int rt = min((row0 >> 5) + fb, a.x_tiles - 1);
    src[2 + p] = a.xp + ((size_t)rt * KC) * 64 + lane;
    dst[2 + p] = lds0 + 16384u + (uint32_t)(fb * 2) * 1024u;
  }
  // one eighth (j) of this wave's copies of stage i: k-tile j % 2 of operand tile row j / 2
  auto copy_one = [&](int i, int slot, int j) {
    const size_t k = (size_t)min(i, n_steps - 1) * 128;  // 2 k-tiles of 64 uint4
    const uint32_t d = dst[j >> 1] + (uint32_t)slot * (T2_STAGE * 16) + (uint32_t)(j & 1) * 1024u;
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, off"
        :
        : "s"(d), "v"(src[j >> 1] + k + (j & 1) * 64)
        : "memory", "m0");
  };
  auto copy_stage = [&](int i) {
#pragma unroll
    for (int j = 0; j < 8; ++j) copy_one(i, i, j);
  };

  constexpr int NX = NA > 0 ? NA : 1;
  f32x16 acc[4][NX];
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int m = 0; m < NX; ++m)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[f][m][i] = 0.f;

  // Fragments of a k-tile: weight blocks 4 wi + f, row tiles 2 m + wj of the block (the two
  // row halves interleave, so that a ragged last block splits evenly).  A wave has one
  // instruction stream and nothing else runs on its SIMD, so whatever is not an MFMA is
  // issued BETWEEN the MFMAs of a k-tile, one piece after each: the LDS reads of the next
  // k-tile's fragments (4 + NA of them) and the eight copies of a stage.
  uint4 W0[4], X0[NX], W1[4], X1[NX];
  auto read_one = [&](const uint4* s, int q, uint4(&Wf)[4], uint4(&Xf)[NX]) {
#pragma unroll
    for (int f = 0; f < 4; ++f)
      if (q == f) Wf[f] = s[(4 * wi + f) * 128];
#pragma unroll
    for (int m = 0; m < NA; ++m)
      if (q == 4 + m) Xf[m] = s[1024 + (2 * m + wj) * 128];
  };

  // Copies in flight: 8 per stage and wave.  When step i needs stage i + 1 (at its barrier)
  // the stages i + 2 .. i + T2_RING - 1 have been asked for behind it: "at most 8 (T2_RING - 2)
  // outstanding" means that this wave's part of stage i + 1 has landed, and the barrier makes
  // that all four parts.  The same barrier says that every wave has read all of stage i (its
  // LDS reads are waited for before it), whose slot the copies of stage i + T2_RING may then
  // overwrite; they are issued during step i + 1.
#pragma unroll
  for (int i = 0; i < T2_RING - 1; ++i) copy_stage(i);
  VLAC_T2_WAIT();
  __syncthreads();
  if constexpr (NA > 0) {
#pragma unroll
    for (int q = 0; q < 4 + NA; ++q) read_one(lds + lane, q, W0, X0);
  }
  int slot = 0;  // i % T2_RING
  for (int i = 0; i < n_steps; ++i) {
    const int slot_next = slot + 1 == T2_RING ? 0 : slot + 1, slot_copy = slot == 0 ? T2_RING - 1 : slot - 1;
    const uint4* cur = lds + slot * T2_STAGE + lane;
    const uint4* nxt = lds + slot_next * T2_STAGE + lane;
    // k-tile 0 of stage i (fragments W0, X0); meanwhile: read k-tile 1, copy stage i + 3
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 4 * NX; ++q) {
      if constexpr (NA > 0) acc[q / NX][q % NX] = mfma32<F16>(W0[q / NX], X0[q % NX], acc[q / NX][q % NX]);
      if constexpr (NA > 0) read_one(cur + 64, q, W1, X1);
      if constexpr (NX >= 2) {  // one copy after each of the last 8 MFMAs
        if (q >= 4 * NX - 8) copy_one(i + T2_RING - 1, slot_copy, q - (4 * NX - 8));
      } else {                  // 4 MFMAs (or none): two copies after each
        copy_one(i + T2_RING - 1, slot_copy, 2 * q);
        copy_one(i + T2_RING - 1, slot_copy, 2 * q + 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (NA > 0) {
#pragma unroll
      for (int q = 4 * NX; q < 4 + NA; ++q) read_one(cur + 64, q, W1, X1);  // (NA = 1: 5 reads, 4 MFMAs)
    }
    // k-tile 1 (W1, X1): its first MFMA covers the barrier; then read k-tile 0 of stage i + 1
    // (past the last step: a stale stage, unused)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 4 * NX; ++q) {
      if constexpr (NA > 0) acc[q / NX][q % NX] = mfma32<F16>(W1[q / NX], X1[q % NX], acc[q / NX][q % NX]);
      if (q == 0) {
        VLAC_T2_WAIT();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
      } else if constexpr (NA > 0) {
        read_one(nxt, q - 1, W0, X0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (NA > 0) {
#pragma unroll
      for (int q = 4 * NX - 1; q < 4 + NA; ++q) read_one(nxt, q, W0, X0);
    }
    slot = slot_next;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no copy outlives the loop

  if constexpr (NA > 0) {
    const int g = lane >> 5;
    if (a.wscale) {  // weights expanded from e4m3 codes: the scale of every output feature
#pragma unroll
      for (int f = 0; f < 4; ++f)
        if (nb0 + 4 * wi + f < a.NB) {
#pragma unroll
          for (int m = 0; m < NA; ++m) scale_tile(a.wscale, nb0 + 4 * wi + f, g, acc[f][m]);
        }
    }
#pragma unroll
    for (int m = 0; m < NA; ++m) {
      const int slot = row0 + (2 * m + wj) * 32 + (lane & 31);
      if (slot < n_rows) {
        const int id = (EPI == EPI_LOGITS) ? 0 : a.e.rows[slot];
#pragma unroll
        for (int f = 0; f < 4; ++f)
          if (nb0 + 4 * wi + f < a.NB) epilogue_tile<EPI, F16>(a.e, nb0 + 4 * wi + f, slot, id, g, acc[f][m]);
      }
    }
  }
}

template <int RT, int EPI, bool F16>
__device__ __forceinline__ void tall2_dispatch(const GemmArgs& a, uint4* lds, int tile, int mb, int n_rows) {
  // row tiles of this block, dealt to the two row halves alternately
  const int nt = min(2 * RT, (n_rows - mb * (64 * RT) + 31) >> 5);
  const int wj = threadIdx.x >> 7;
  const int na = (nt - wj + 1) >> 1;  // wave-uniform
  if constexpr (RT == 4) {
    switch (na) {
      case 0: tall2_body<4, 0, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 1: tall2_body<4, 1, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 2: tall2_body<4, 2, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 3: tall2_body<4, 3, EPI, F16>(a, lds, tile, mb, n_rows); break;
      default: tall2_body<4, 4, EPI, F16>(a, lds, tile, mb, n_rows); break;
    }
  } else if constexpr (RT == 3) {
    switch (na) {
      case 0: tall2_body<3, 0, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 1: tall2_body<3, 1, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 2: tall2_body<3, 2, EPI, F16>(a, lds, tile, mb, n_rows); break;
      default: tall2_body<3, 3, EPI, F16>(a, lds, tile, mb, n_rows); break;
    }
  } else {
    switch (na) {
      case 0: tall2_body<2, 0, EPI, F16>(a, lds, tile, mb, n_rows); break;
      case 1: tall2_body<2, 1, EPI, F16>(a, lds, tile, mb, n_rows); break;
      default: tall2_body<2, 2, EPI, F16>(a, lds, tile, mb, n_rows); break;
    }
  }
}

template <int EPI, bool F16>
__global__ __launch_bounds__(256) void gemm_tall2_kernel(GemmArgs a) {
  extern __shared__ uint4 lds[];  // T2_RING stages of 32 KiB
  // Work items are (weight tile, row block) pairs, listed with the row blocks of one weight
  // tile next to each other, and the list is cut into eight equal runs, one per XCD
  // (workgroup id % 8), so that the row blocks of a weight tile share it in one L2 and every
  // XCD gets the same number of items.  The grid covers the most items any row count can
  // give; the items of the actual row count come first in every XCD's run.
  const int n_rows = a.n_rows_val >= 0 ? a.n_rows_val : *a.n_rows;
  if (n_rows < a.rows_lo) return;  // the one-stream kernel's share
  const Tall2Plan pl = tall2_plan((a.NB + 7) >> 3, n_rows);
  const int items = pl.tiles * pl.row_blocks, per = (items + 7) >> 3;
  const int j = blockIdx.x >> 3, i = (blockIdx.x & 7) * per + j;
  if (j >= per || i >= items) return;
  const int tile = i / pl.row_blocks, mb = i - tile * pl.row_blocks;
  if (pl.rt == 4) tall2_dispatch<4, EPI, F16>(a, lds, tile, mb, n_rows);
  else if (pl.rt == 3) tall2_dispatch<3, EPI, F16>(a, lds, tile, mb, n_rows);
  else tall2_dispatch<2, EPI, F16>(a, lds, tile, mb, n_rows);
}

template <int EPI, bool F16>
hipError_t set_lds() {
  return hipFuncSetAttribute((const void*)gemm_tall2_kernel<EPI, F16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             T2_RING * T2_STAGE * 16);
}

template <bool F16>
void launch_tall2_t(int epi, const GemmArgs& a, int grid, hipStream_t st) {
  const size_t shm = (size_t)T2_RING * T2_STAGE * 16;
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_tall2_kernel<EPI_QKV, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_tall2_kernel<EPI_SWIGLU, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_tall2_kernel<EPI_LOGITS, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
  }
}

}  // namespace

int gemm_tall2_init() {
  hipError_t e;
  if ((e = set_lds<EPI_QKV, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_QKV, false>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_SWIGLU, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_SWIGLU, false>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_LOGITS, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_LOGITS, false>()) != hipSuccess) return (int)e;
  return 0;
}

void launch_gemm_tall2(bool f16, int epi, GemmArgs& a, int rows_cap, hipStream_t st) {
  a.S = 1;
  a.MB = (rows_cap + 127) / 128;
  a.P = 0;
  a.x_tiles = (rows_cap + 31) / 32;
  // the grid covers the most work items any row count up to rows_cap can give (the plan
  // changes its row blocks with the row count)
  const int tiles = (a.NB + 7) >> 3;
  int most = 0;
  for (int n = 64; n < rows_cap + 64; n += 64) most = std::max(most, tall2_plan(tiles, std::min(n, rows_cap)).items());
  const int grid = ((most + 7) / 8) * 8;
  if (f16) launch_tall2_t<true>(epi, a, grid, st);
  else launch_tall2_t<false>(epi, a, grid, st);
}
