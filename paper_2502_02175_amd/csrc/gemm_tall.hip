// Recomputed-row GEMMs with MANY rows (batched streams: thousands of rows per layer;
// Alg. 2 of VLA-Cache over the rows outside P_reuse of every stream at once).
//
// With thousands of rows the weights are no longer the traffic: the GEMM is bound by the
// matrix cores, and behind them by what reaches a CU from L2 (measured here: 20 to 27 bytes
// per clock and CU), so the operand bytes fetched per MFMA are what has to be kept small.
// A work item is 256 features x 256 rows (16 KiB of operands per 64 MFMAs), and both operand
// tiles are shared through LDS:
//
//  * 4 waves, one per SIMD; a wave owns 4 feature blocks x 4 row tiles = 16 accumulator
//    tiles (256 accumulator registers), and one k-tile is 16 MFMAs for 8 operand fragments
//    read from LDS.
//  * Operands are in fragment order (common.h): a tile is 1 KiB that a wave copies global ->
//    LDS as it lies (global_load_lds_dwordx4: lane l's 16 bytes land at base + 16 l) and
//    reads back with one 16-byte LDS read per lane, conflict-free.
//  * A stage is 32 k: 16 weight tiles + 16 activation tiles = 32 KiB; a ring of 5 stages
//    (all 160 KiB of a CU's LDS), copies run 4 stages ahead.  Every wave copies 8 tiles per
//    stage, whatever the row count (tiles past the end are clamped to a valid one and never
//    read), so that the number of copies in flight is the same for every wave at every step:
//    the copies are inline assembly that the compiler does not see (it treats its own
//    LDS-direct loads as aliasing every LDS read and drains the load queue at each), and
//    their waits are placed by hand (VLAC_VMCNT; a build with -DVLAC_SAFE_WAITS waits for
//    everything instead and must give the same bits).
//  * One barrier per stage, placed behind the first MFMA of its second k-tile: the fragments
//    of a k-tile are read while the MFMAs of the one before run, across the barrier as well.
//  * The grid is one workgroup per CU; a workgroup runs its work items one after the other
//    and copies the first stages of the next item during the last steps of the one before.
//  * Row blocks of 192 or 128 rows (a wave owns 4 x 3 or 4 x 2 tiles), and K split in 2 or 3
//    parts in the projections with a residual (whose consumer, residual add + RMSNorm, adds
//    the partial rows up), where that takes less time by the estimate of tall_plan, which
//    kernel and consumer evaluate on the device from the actual row count.
//  * Measured against this design and not kept: a 512-feature x 128-row item with the weight
//    tiles fetched global -> registers by 8 waves (20 KiB per 64 MFMAs: 5 to 8 % slower at
//    the 7B layer shape with 2700 to 8400 rows, equal at d_model 1536); rings of 4 stages
//    (equal); all copies of a stage issued together instead of one per MFMA (7 % slower: a
//    wave's copies and LDS reads hold up its own MFMAs); hardware dispatch of one workgroup
//    per item (equal at K 4096, 5 % slower at K 1536, where an item is short).  With the
//    copies or the LDS reads taken out (wrong results, timing only) the gate/up GEMM at 2712
//    rows goes from 440 to 362 and 422 us, with both out to 346 us: the matrix cores
//    themselves, with one barrier per stage and the last of 3.7 rounds of items a partial
//    one, do not get past 0.57 of the published peak on this chip.
#include "gemm_epi.h"

namespace {

#ifndef VLAC_TALL_RING
#define VLAC_TALL_RING 5
#endif
constexpr int TALL_RING = VLAC_TALL_RING;  // LDS stages: 5 x 32 KiB is all the LDS of a CU
// copies younger than the stage a step waits for: those of the TALL_RING - 2 stages behind it
#if VLAC_TALL_RING == 5
#define VLAC_TALL_WAIT() VLAC_VMCNT(24)
#elif VLAC_TALL_RING == 4
#define VLAC_TALL_WAIT() VLAC_VMCNT(16)
#else
#error "add the wait for this ring size"
#endif
constexpr int TALL_STAGE = 2048;        // uint4 per stage: 32 tiles of 64
constexpr int kTallGrid = 256;          // one workgroup per CU (a workgroup takes all of a CU's LDS)

// A work item: weight tile, K part, row block
struct TallItem { int tile, s, mb; };

// RT: row tiles per wave (4: blocks of 256 rows, 3: of 192, 2: of 128); NA: how many of them hold rows.
// Runs item `it`; `nx` is the item this workgroup runs next (chain: there is one, and the last
// TALL_RING - 1 steps of this item copy its first stages instead of stages past the end).
// prefilled: the copies of this item's first TALL_RING - 1 stages have been issued already (by
// the item before) into the ring from `slot` on.  Returns the ring slot after the last stage.
template <int RT, int NA, int EPI, bool F16>
__device__ __forceinline__ int tall_body(const GemmArgs& a, uint4* lds, TallItem it, TallItem nx, bool chain,
                                          bool prefilled, int slot, int n_rows, int S) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = w & 1, wj = w >> 1;  // feature half, row interleave
  const int KC = 4 * a.KS;
  // part s of S of the 32-k steps of K
  const int sq = (2 * a.KS) / S, sr = (2 * a.KS) % S;
  const int step0 = it.s * sq + min(it.s, sr), n_steps = sq + (it.s < sr ? 1 : 0);
  const int step0n = nx.s * sq + min(nx.s, sr), n_steps_n = sq + (nx.s < sr ? 1 : 0);
  const int row0 = it.mb * (64 * RT);
  const int nb0 = it.tile * 8;
  // This wave copies, per stage, the weight tiles of feature blocks 2w, 2w + 1 and the
  // activation tiles of row tiles 2w, 2w + 1 of the block (both k-tiles of each: 2 KiB that
  // lie together in global memory and in LDS).  Row blocks of 128 rows have 4 row tiles:
  // waves 2 and 3 copy tiles 4..7 all the same (clamped, unread).
  // (scalar base addresses: a copy is then one scalar select, one scalar add and the load, with
  // the lane's 16-byte offset in one register for all of them; a wave has one instruction stream,
  // and what a copy costs to issue is taken from its MFMAs)
  const char *src[4], *srcn[4];
  uint32_t dst[4];
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds);
  const uint32_t lane_off = (uint32_t)lane * 16u;
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int fb = 2 * w + p;
    src[p] = (const char*)(a.wp + ((size_t)min(nb0 + fb, a.NB - 1) * KC + 2 * step0) * 64);
    srcn[p] = (const char*)(a.wp + ((size_t)min(nx.tile * 8 + fb, a.NB - 1) * KC + 2 * step0n) * 64);
    dst[p] = lds0 + (uint32_t)(fb * 2) * 1024u;
    src[2 + p] = (const char*)(a.xp + ((size_t)min((row0 >> 5) + fb, a.x_tiles - 1) * KC + 2 * step0) * 64);
    srcn[2 + p] = (const char*)(a.xp + ((size_t)min(nx.mb * (2 * RT) + fb, a.x_tiles - 1) * KC + 2 * step0n) * 64);
    dst[2 + p] = lds0 + 16384u + (uint32_t)(fb * 2) * 1024u;
  }
  // one eighth (j) of this wave's copies of stage i: k-tile j % 2 of operand tile row j / 2.
  // Stages past this item's last are the next item's first (chain), else its last again
  // (never read): the number of copies per step is the same at every step.
  auto copy_one = [&](int i, int slot_, int j) {
    const bool mine = i < n_steps || !chain;
    const size_t k = (size_t)(mine ? min(i, n_steps - 1) : min(i - n_steps, n_steps_n - 1)) * 2048;  // 2 k-tiles of 1 KiB
    const char* sp = (mine ? src[j >> 1] : srcn[j >> 1]) + k + (j & 1) * 1024;
    const uint32_t d = dst[j >> 1] + (uint32_t)slot_ * (TALL_STAGE * 16) + (uint32_t)(j & 1) * 1024u;
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2"
        :
        : "s"(d), "v"(lane_off), "s"(sp)
        : "memory", "m0");
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
  // the stages i + 2 .. i + TALL_RING - 1 have been asked for behind it: "at most 8 (TALL_RING - 2)
  // outstanding" means that this wave's part of stage i + 1 has landed, and the barrier makes
  // that all four parts.  The same barrier says that every wave has read all of stage i (its
  // LDS reads are waited for before it), whose slot the copies of stage i + TALL_RING may then
  // overwrite; they are issued during step i + 1.  Stages are numbered on through a chain of
  // items, so all of this holds across the item boundary as well: the barrier of an item's
  // last step is the one that waits for the next item's stage 0.  (Other vector-memory
  // operations of the wave, the epilogue's, are all younger or all older than the copies a
  // step waits for; loads return in issue order, so they can only make a wait longer.)
  if (!prefilled) {
    int sl = slot;
#pragma unroll
    for (int i = 0; i < TALL_RING - 1; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) copy_one(i, sl, j);
      sl = sl + 1 == TALL_RING ? 0 : sl + 1;
    }
    VLAC_TALL_WAIT();
    __syncthreads();
  }
  if constexpr (NA > 0) {
#pragma unroll
    for (int q = 0; q < 4 + NA; ++q) read_one(lds + slot * TALL_STAGE + lane, q, W0, X0);
  }
  for (int i = 0; i < n_steps; ++i) {
    const int slot_next = slot + 1 == TALL_RING ? 0 : slot + 1, slot_copy = slot == 0 ? TALL_RING - 1 : slot - 1;
    const uint4* cur = lds + slot * TALL_STAGE + lane;
    const uint4* nxt = lds + slot_next * TALL_STAGE + lane;
    // k-tile 0 of stage i (fragments W0, X0); meanwhile: read k-tile 1, copy stage i + TALL_RING - 1
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 4 * NX; ++q) {
      if constexpr (NA > 0) acc[q / NX][q % NX] = mfma32<F16>(W0[q / NX], X0[q % NX], acc[q / NX][q % NX]);
      if constexpr (NA > 0) read_one(cur + 64, q, W1, X1);
      if constexpr (NX >= 2) {  // one copy after each of the last 8 MFMAs
        if (q >= 4 * NX - 8) copy_one(i + TALL_RING - 1, slot_copy, q - (4 * NX - 8));
      } else {                  // 4 MFMAs (or none): two copies after each
        copy_one(i + TALL_RING - 1, slot_copy, 2 * q);
        copy_one(i + TALL_RING - 1, slot_copy, 2 * q + 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (NA > 0) {
#pragma unroll
      for (int q = 4 * NX; q < 4 + NA; ++q) read_one(cur + 64, q, W1, X1);  // (NA = 1: 5 reads, 4 MFMAs)
    }
    // k-tile 1 (W1, X1): its first MFMA covers the barrier; then read k-tile 0 of stage i + 1
    // (after the last step: of a stage that is not this item's; the next item reads its own)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 4 * NX; ++q) {
      if constexpr (NA > 0) acc[q / NX][q % NX] = mfma32<F16>(W1[q / NX], X1[q % NX], acc[q / NX][q % NX]);
      if (q == 0) {
        VLAC_TALL_WAIT();
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
  if (!chain) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no copy outlives the item
    __syncthreads();                                  // (the next item's copies overwrite any slot)
  }

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
    if (EPI == EPI_RESID && S > 1) {
      // split K: the partial rows [part][row][feature] are left to the row kernel that follows
      // (residual add + RMSNorm), which adds the parts up in order
#pragma unroll
      for (int m = 0; m < NA; ++m) {
        const int slot_r = row0 + (2 * m + wj) * 32 + (lane & 31);
        if (slot_r < n_rows) {
#pragma unroll
          for (int f = 0; f < 4; ++f)
            if (nb0 + 4 * wi + f < a.NB) {
              float* dp = a.e.rpart + ((size_t)it.s * a.e.rpart_rows + slot_r) * a.e.d_model + (nb0 + 4 * wi + f) * 32 + 4 * g;
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4)
                *(float4*)(dp + 8 * q4) = make_float4(acc[f][m][4 * q4], acc[f][m][4 * q4 + 1],
                                                      acc[f][m][4 * q4 + 2], acc[f][m][4 * q4 + 3]);
            }
        }
      }
    } else {
#pragma unroll
      for (int m = 0; m < NA; ++m) {
        const int slot_r = row0 + (2 * m + wj) * 32 + (lane & 31);
        if (slot_r < n_rows) {
          const int id = (EPI == EPI_LOGITS) ? 0 : a.e.rows[slot_r];
#pragma unroll
          for (int f = 0; f < 4; ++f)
            if (nb0 + 4 * wi + f < a.NB) epilogue_tile<EPI, F16>(a.e, nb0 + 4 * wi + f, slot_r, id, g, acc[f][m]);
        }
      }
    }
  }
  return slot;
}

template <int RT, int EPI, bool F16>
__device__ __forceinline__ int tall_dispatch(const GemmArgs& a, uint4* lds, TallItem it, TallItem nx, bool chain,
                                              bool prefilled, int slot, int n_rows, int S) {
  // row tiles of this block, dealt to the two row halves alternately
  const int nt = min(2 * RT, (n_rows - it.mb * (64 * RT) + 31) >> 5);
  const int wj = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7);
  const int na = (nt - wj + 1) >> 1;  // wave-uniform
#define VLAC_TALL_CASE(N) case N: return tall_body<RT, N, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, S);
  switch (na) {
    VLAC_TALL_CASE(0)
    VLAC_TALL_CASE(1)
    VLAC_TALL_CASE(2)
    default:
      if constexpr (RT == 2) return tall_body<RT, 2, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, S);
      else if constexpr (RT == 3) return tall_body<RT, 3, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, S);
      else {
        if (na == 3) return tall_body<RT, 3, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, S);
        return tall_body<RT, 4, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, S);
      }
  }
#undef VLAC_TALL_CASE
}

template <int RT, int EPI, bool F16>
__device__ __forceinline__ void tall_items(const GemmArgs& a, uint4* lds, const TallPlan& pl, int n_rows) {
  // Work items are (weight tile, K part, row block) triples, listed with the row blocks of one
  // weight tile and part next to each other, and the list is cut into eight equal runs, one
  // per XCD (workgroup id % 8), so that the row blocks of a weight tile share it in one L2 and
  // every XCD gets the same number of items.  The grid is one workgroup per CU; a workgroup
  // takes every (grid / 8)-th item of its XCD's run, one after the other, and starts the
  // copies of its next item's first stages during the last steps of the one before it, so
  // that only a workgroup's first item waits for its operands.
  const int items = pl.items(), per = (items + 7) >> 3;
  const int x = blockIdx.x & 7, stride = gridDim.x >> 3;
  auto item_of = [&](int j) {
    const int i = x * per + j;
    const int vt = i / pl.row_blocks;
    TallItem t;
    t.mb = i - vt * pl.row_blocks;
    t.tile = vt / pl.S;
    t.s = vt - t.tile * pl.S;
    return t;
  };
  auto exists = [&](int j) { return j < per && x * per + j < items; };
  int j = blockIdx.x >> 3;
  if (!exists(j)) return;
  // (chains need every part of K to have at least as many steps as the copies run ahead)
  const bool can_chain = (2 * a.KS) / pl.S >= TALL_RING - 1;
  TallItem it = item_of(j);
  bool prefilled = false;
  int slot = 0;
  for (;;) {
    const int jn = j + stride;
    const bool chain = can_chain && exists(jn);
    const TallItem nx = chain ? item_of(jn) : it;
    slot = tall_dispatch<RT, EPI, F16>(a, lds, it, nx, chain, prefilled, slot, n_rows, pl.S);
    if (!exists(jn)) break;
    prefilled = chain;
    it = item_of(jn);
    j = jn;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <int EPI, bool F16>
__global__ __launch_bounds__(256) void gemm_tall_kernel(GemmArgs a) {
  extern __shared__ uint4 lds[];  // TALL_RING stages of 32 KiB
  const int n_rows = a.n_rows_val >= 0 ? a.n_rows_val : *a.n_rows;
  if (n_rows < a.rows_lo) return;  // the one-stream kernel's share
  const TallPlan pl = tall_plan((a.NB + 7) >> 3, n_rows, EPI == EPI_RESID ? a.S : 1, a.KS);
  if (pl.rt == 4) tall_items<4, EPI, F16>(a, lds, pl, n_rows);
  else if (pl.rt == 3) tall_items<3, EPI, F16>(a, lds, pl, n_rows);
  else tall_items<2, EPI, F16>(a, lds, pl, n_rows);
}

template <int EPI, bool F16>
hipError_t set_lds() {
  return hipFuncSetAttribute((const void*)gemm_tall_kernel<EPI, F16>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             TALL_RING * TALL_STAGE * 16);
}

template <bool F16>
void launch_tall_t(int epi, const GemmArgs& a, int grid, hipStream_t st) {
  const size_t shm = (size_t)TALL_RING * TALL_STAGE * 16;
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_QKV, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_SWIGLU, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_RESID:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_RESID, F16>), dim3(grid), dim3(256), shm, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_tall_kernel<EPI_LOGITS, F16>), dim3(grid), dim3(256), shm, st, a);
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

int gemm_tall_init() {
  hipError_t e;
  if ((e = set_lds<EPI_QKV, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_QKV, false>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_SWIGLU, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_SWIGLU, false>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_RESID, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_RESID, false>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_LOGITS, true>()) != hipSuccess) return (int)e;
  if ((e = set_lds<EPI_LOGITS, false>()) != hipSuccess) return (int)e;
  return 0;
}

void launch_gemm_tall(bool f16, int epi, GemmArgs& a, int rows_cap, int S_max, hipStream_t st) {
  a.S = (epi == EPI_RESID && S_max > 1) ? S_max : 1;
  a.MB = (rows_cap + 127) / 128;
  a.P = 0;
  a.x_tiles = (rows_cap + 31) / 32;
  // the grid covers the most work items any row count up to rows_cap can give (the plan
  // changes its row blocks and K parts with the row count)
  const int tiles = (a.NB + 7) >> 3;
  int most = 0;
  for (int n = 64; n < rows_cap + 64; n += 64)
    most = std::max(most, tall_plan(tiles, std::min(n, rows_cap), a.S, a.KS).items());
  const int grid = std::min(((most + 7) / 8) * 8, kTallGrid);
  if (f16) launch_tall_t<true>(epi, a, grid, st);
  else launch_tall_t<false>(epi, a, grid, st);
}
