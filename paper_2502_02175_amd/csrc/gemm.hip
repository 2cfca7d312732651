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
//    v_mfma_f32_32x32x16_{bf16,f16} without any shuffling.
//  * The matrix-core A operand is the WEIGHT tile (32 output features x 16 k),
//    the B operand the activation tile (16 k x 32 rows); a lane of the result
//    holds one row and 4 x 4 consecutive features, which is what the fused
//    epilogues want (rotary partners, gate/up pairs and packed 8-byte stores in
//    one lane).
//  * A workgroup is 4 waves = 4 x 32 output features over all rows of its row
//    block (4 tiles of 32 rows, accumulators in registers; more rows = more row
//    blocks, mapped to the same XCD so that they share the weight tiles in L2).  Weight tiles go
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
#include <cstring>
#include "gemm_epi.h"

// Main loop, split-K hand-over and epilogue for a row block with exactly NA active
// 32-row tiles (a template parameter, so that every loop is unrolled without guards
// and the compiler can count the loads in flight exactly).
template <int NA, int MT, int EPI, bool F16, bool W8>
__device__ __forceinline__ void rows_body(const GemmArgs& a, uint4* lds, int* s_last, int tile,
                                          int s, int mb, int n_rows, uint32_t pf0, uint32_t pf1) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int row0 = mb * MT * 32;
  const int nb = tile * 4 + w;
  const bool wave_on = nb < a.NB;
  const int KC = 4 * a.KS;
  const int q = a.KS / a.S, r = a.KS % a.S;
  const int ks0 = s * q + min(s, r), n_ks = q + (s < r ? 1 : 0);
  // (e4m3 weights: a 16-byte lane slot holds two k-tiles, a step is two slots per wave)
  const uint4* wsrc = a.wp + ((size_t)(wave_on ? nb : a.NB - 1) * (W8 ? KC / 2 : KC) + (W8 ? 2 : 4) * ks0) * 64 + lane;
  const uint4* xsrc = a.xp + ((size_t)(row0 >> 5) * KC + 4 * ks0) * 64 + tid;

  f32x16 acc[NA];
#pragma unroll
  for (int mt = 0; mt < NA; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
  // Register stages as individually named variables (arrays of them end up in scratch
  // memory): weight tiles (B0..B3) and activation tiles (A0..A3) of four steps each.
  // Loads return in issue order, so a tile can only be consumed once everything issued
  // before it has landed: the L2-resident activation tiles must be fetched as far ahead
  // as the HBM-resident weight tiles, or they would wait behind them at every step.
  uint4 B0_0, B0_1, B0_2, B0_3, B1_0, B1_1, B1_2, B1_3, B2_0, B2_1, B2_2, B2_3, B3_0, B3_1, B3_2, B3_3;
  uint4 A0_0, A0_1, A0_2, A0_3, A1_0, A1_1, A1_2, A1_3, A2_0, A2_1, A2_2, A2_3, A3_0, A3_1, A3_2, A3_3;
  A0_1 = A0_2 = A0_3 = A1_1 = A1_2 = A1_3 = make_uint4(0, 0, 0, 0);
  A2_1 = A2_2 = A2_3 = A3_1 = A3_2 = A3_3 = make_uint4(0, 0, 0, 0);

  // step i of this workgroup covers k-tiles 4i .. 4i+3 of its K range
#define VLAC_LOAD_B(i, P)                                   \
  {                                                         \
    const size_t k_ = (size_t)min((i), n_ks - 1) * (W8 ? 128 : 256); \
    P##_0 = wsrc[k_];                                       \
    P##_1 = wsrc[k_ + 64];                                  \
    if constexpr (!W8) {                                    \
      P##_2 = wsrc[k_ + 128];                               \
      P##_3 = wsrc[k_ + 192];                               \
    }                                                       \
  }
#define VLAC_LOAD_A(i, P)                                             \
  {                                                                   \
    const size_t k_ = (size_t)min((i), n_ks - 1) * 256;               \
    P##_0 = xsrc[k_];                                                 \
    if constexpr (NA > 1) P##_1 = xsrc[(size_t)KC * 64 + k_];         \
    if constexpr (NA > 2) P##_2 = xsrc[(size_t)KC * 128 + k_];        \
    if constexpr (NA > 3) P##_3 = xsrc[(size_t)KC * 192 + k_];        \
  }
#define VLAC_STORE_A(buf, P)                                                  \
  {                                                                           \
    lds[((buf) * MT + 0) * 256 + tid] = P##_0;                                \
    if constexpr (NA > 1) lds[((buf) * MT + 1) * 256 + tid] = P##_1;          \
    if constexpr (NA > 2) lds[((buf) * MT + 2) * 256 + tid] = P##_2;          \
    if constexpr (NA > 3) lds[((buf) * MT + 3) * 256 + tid] = P##_3;          \
  }
#define VLAC_MMA(c, BW)                                                       \
  _Pragma("unroll") for (int mt = 0; mt < NA; ++mt) acc[mt] =                 \
      mfma32<F16>(BW, lds[(buf_ * MT + mt) * 256 + (c) * 64 + lane], acc[mt]);
  // the weight tile of k-tile c of a step: a register of its own, or half of a slot of codes
#define VLAC_MMA4(P)                                                                          \
  if constexpr (W8) {                                                                         \
    const uint4 w0_ = e4m3_slot_half(B##P##_0, 0), w1_ = e4m3_slot_half(B##P##_0, 1);         \
    const uint4 w2_ = e4m3_slot_half(B##P##_1, 0), w3_ = e4m3_slot_half(B##P##_1, 1);         \
    VLAC_MMA(0, w0_) VLAC_MMA(1, w1_) VLAC_MMA(2, w2_) VLAC_MMA(3, w3_)                       \
  } else {                                                                                    \
    VLAC_MMA(0, B##P##_0) VLAC_MMA(1, B##P##_1) VLAC_MMA(2, B##P##_2) VLAC_MMA(3, B##P##_3)   \
  }
  // Step i: stage slot P held step i (its activation tiles went to LDS during step i-1,
  // its weight tiles are consumed now) and is refilled with step i+4; the activation
  // tiles of step i+1 (slot PN) go to the other LDS buffer.  The phases are fenced
  // against the instruction scheduler so that loads are issued in this order.
#define VLAC_STEP(i, P, PN)                                                   \
  {                                                                           \
    const int buf_ = (i) & 1;                                                 \
    __syncthreads();                                                          \
    VLAC_LOAD_A((i) + 4, A##P)                                                \
    __builtin_amdgcn_sched_barrier(0);                                        \
    VLAC_MMA4(P)                                                              \
    __builtin_amdgcn_sched_barrier(0);                                        \
    VLAC_LOAD_B((i) + 4, B##P)                                                \
    __builtin_amdgcn_sched_barrier(0);                                        \
    VLAC_STORE_A(buf_ ^ 1, A##PN)                                             \
  }

  VLAC_LOAD_A(0, A0) VLAC_LOAD_B(0, B0)
  VLAC_LOAD_A(1, A1) VLAC_LOAD_B(1, B1)
  VLAC_LOAD_A(2, A2) VLAC_LOAD_B(2, B2)
  VLAC_LOAD_A(3, A3) VLAC_LOAD_B(3, B3)
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::"v"(pf0), "v"(pf1));  // the touch loads end here, behind the real ones
  VLAC_STORE_A(0, A0)
  // Whole groups of 4 steps run in a loop without any branch inside (a conditional step
  // would make the compiler assume the shortest path around the loop and wait for almost
  // every load at the top of each iteration); the 0..3 remaining steps follow.
  int i0 = 0;
  for (; i0 + 4 <= n_ks; i0 += 4) {
    VLAC_STEP(i0, 0, 1)
    VLAC_STEP(i0 + 1, 1, 2)
    VLAC_STEP(i0 + 2, 2, 3)
    VLAC_STEP(i0 + 3, 3, 0)
  }
  if (i0 < n_ks) {
    VLAC_STEP(i0, 0, 1)
    if (i0 + 1 < n_ks) {
      VLAC_STEP(i0 + 1, 1, 2)
      if (i0 + 2 < n_ks) VLAC_STEP(i0 + 2, 2, 3)
    }
  }
#undef VLAC_MMA4
#undef VLAC_MMA
#undef VLAC_STEP
#undef VLAC_STORE_A
#undef VLAC_LOAD_A
#undef VLAC_LOAD_B

  if constexpr (W8) {
    if (wave_on) {
#pragma unroll
      for (int mt = 0; mt < NA; ++mt) scale_tile(a.wscale, nb, lane >> 5, acc[mt]);
    }
  }
  if (EPI == EPI_RESID && a.S > 1) {
    // Projection + residual with split K: every split writes its partial rows
    // [split][row][feature] and is done; the row kernel that follows (residual add +
    // RMSNorm) adds the splits up, so nothing is handed over inside this kernel.
    if (!wave_on) return;
    const int g = lane >> 5;
#pragma unroll
    for (int mt = 0; mt < NA; ++mt) {
      const int slot = row0 + mt * 32 + (lane & 31);
      if (slot < n_rows) {
        float* dst = a.e.rpart + ((size_t)s * a.e.rpart_rows + slot) * a.e.d_model + nb * 32 + 4 * g;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *(float4*)(dst + 8 * q4) = make_float4(acc[mt][4 * q4], acc[mt][4 * q4 + 1],
                                                 acc[mt][4 * q4 + 2], acc[mt][4 * q4 + 3]);
      }
    }
    return;
  }
  if (a.S > 1) {
    // split-K: park the partial sums; the last workgroup of this (tile, row block) adds them up
    const size_t per_wave = (size_t)MT * 16 * 64;
    float* base = a.partial + ((size_t)(tile * a.MB + mb) * a.S) * 4 * per_wave;
    float* mine = base + ((size_t)s * 4 + w) * per_wave + lane;
#pragma unroll
    for (int mt = 0; mt < NA; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) st_coherent(mine + (mt * 16 + i) * 64, acc[mt][i]);
    stores_done();
    __syncthreads();
    if (tid == 0) {
      int* cnt = a.counters + tile * a.MB + mb;
      const int old = atomicAdd(cnt, 1);
      *s_last = (old == a.S - 1);
      if (old == a.S - 1) *cnt = 0;  // ready for the next launch
    }
    __syncthreads();
    if (!*s_last) return;
#pragma unroll
    for (int mt = 0; mt < NA; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;
    for (int ss = 0; ss < a.S; ++ss) {  // fixed order; a whole split's worth of loads in flight
      const float* src = base + ((size_t)ss * 4 + w) * per_wave + lane;
      float t[NA][16];
#pragma unroll
      for (int mt = 0; mt < NA; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) t[mt][i] = ld_coherent(src + (mt * 16 + i) * 64);
#pragma unroll
      for (int mt = 0; mt < NA; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mt][i] += t[mt][i];
    }
  }

  if (!wave_on) return;
  const int g = lane >> 5;
#pragma unroll
  for (int mt = 0; mt < NA; ++mt) {
    const int slot = row0 + mt * 32 + (lane & 31);
    if (slot < n_rows) {
      const int id = (EPI == EPI_LOGITS) ? 0 : a.e.rows[slot];
      epilogue_tile<EPI, F16>(a.e, nb, slot, id, g, acc[mt]);
    }
  }
}

template <int MT, int EPI, bool F16, bool W8>
__global__ __launch_bounds__(256) void gemm_rows_kernel(GemmArgs a) {
  extern __shared__ uint4 lds[];  // [2][MT][256]: two stages of MT activation tiles x 4 k-tiles
  __shared__ int s_last;
  // workgroup id -> (row block, weight tile, split); id % 8 is the XCD.  With the row
  // count known on the host every row block has work, and the blocks of one weight tile
  // sit next to each other.  Otherwise the grid covers the largest possible row count,
  // and the row block is the slowest index: the workgroups of empty row blocks (which
  // only find that out from device memory) would else sit between the working ones in
  // dispatch order and hold their places.  (Measured: that pays when one row block's
  // workgroups fit on the chip at once, P <= 256; with more, the staggered start of the
  // interleaved order is the better one.)
  int mb, p;
  if (a.n_rows_val >= 0 || a.P > 256) {
    const int y = blockIdx.x >> 3;
    mb = y % a.MB;
    p = (y / a.MB) * 8 + (blockIdx.x & 7);
  } else {
    const int p8 = (a.P + 7) & ~7;
    mb = blockIdx.x / p8;
    p = blockIdx.x - mb * p8;
  }
  if (p >= a.P) return;
  const int tile = p / a.S, s = p - tile * a.S;
  // The row count sits in device memory, and nothing can be loaded into registers before
  // it is known (the loop is specialised by it).  The first row block, which always has
  // work, touches the first 16 KiB of every wave's weight stream meanwhile (one dword per
  // 128-byte line), so that the stream starts from L2 one round trip later.
  uint32_t pf0 = 0, pf1 = 0;
  if (mb == 0 && a.n_rows_val < 0) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, nb = min(tile * 4 + w, a.NB - 1);
    const int q = a.KS / a.S, r = a.KS % a.S;
    const int ks0 = s * q + min(s, r), n_ks = q + (s < r ? 1 : 0);
    if (n_ks >= 4) {
      const uint32_t* pw = (const uint32_t*)(a.wp + ((size_t)nb * 4 * a.KS + 4 * ks0) * (W8 ? 32 : 64)) + lane * 32;
      pf0 = pw[0];
      pf1 = pw[W8 ? 0 : 2048];
    }
  }
  const int n_rows = a.n_rows_val >= 0 ? a.n_rows_val : *a.n_rows;
  const int row0 = mb * MT * 32;
  if (row0 >= n_rows || n_rows >= a.rows_hi) return;  // (rows_hi and more: the many-rows kernel's share)
  static_assert(MT == 4, "row blocks are 4 tiles of 32 rows");
  switch (min(MT, (n_rows - row0 + 31) >> 5)) {
    case 1: rows_body<1, MT, EPI, F16, W8>(a, lds, &s_last, tile, s, mb, n_rows, pf0, pf1); break;
    case 2: rows_body<2, MT, EPI, F16, W8>(a, lds, &s_last, tile, s, mb, n_rows, pf0, pf1); break;
    case 3: rows_body<3, MT, EPI, F16, W8>(a, lds, &s_last, tile, s, mb, n_rows, pf0, pf1); break;
    default: rows_body<4, MT, EPI, F16, W8>(a, lds, &s_last, tile, s, mb, n_rows, pf0, pf1); break;
  }
}

// ---------------------------------------------------------------------------
// At most 32 rows (the decode passes, the output head): one 32-feature block
// per workgroup, the 4 waves split its K range and add up through LDS, so the
// main loop has no barrier and no LDS traffic at all: every wave streams its
// own contiguous run of weight tiles, two batches of 8 KiB in flight, and reads
// the matching activation tiles straight from L2 (only the lanes of real rows
// load anything).  With S > 1 the K range is also split over S workgroups
// (N = d_model gives only d/32 blocks); the partial tiles are 4 KiB each.
// Where the input is the residual stream and there are at most 4 rows, its RMSNorm is
// done here as well: every workgroup normalises the rows itself (from L2, while its first
// weight tiles are in flight) and keeps the operand slices of its K range in LDS, which
// saves a launch per GEMM in the decode loop.  Split-K partial rows that the previous
// projection left behind are added to the rows on the way (in a fixed order, the same in
// every workgroup), and workgroup 0 stores the completed rows for the next projection.
// ---------------------------------------------------------------------------
// XMODE: where the row operand comes from.
//   X_GLOBAL  every lane loads its 16 bytes of the 32-row operand tile from L2 (any row count)
//   X_NORM4/8 RMSNorm of fp32 rows of at most 4096 / 8192 elements, slices [k/8][row] in LDS
enum { X_GLOBAL = 0, X_NORM4 = 1, X_NORM8 = 2 };

template <int EPI, bool F16, int XMODE, bool W8>
__global__ __launch_bounds__(256, XMODE == X_NORM8 ? 2 : 3) void gemm_few_kernel(GemmArgs a) {
  __shared__ float red[3][16][64];
  extern __shared__ uint4 xlds[];  // operand slices [k/8 - lo8][row]
  constexpr int U = 8;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nb = blockIdx.x / a.S, s = blockIdx.x - nb * a.S;
  const int n_rows = min(a.n_rows_val >= 0 ? a.n_rows_val : *a.n_rows, 32);
  if (n_rows <= 0) return;
  const int KC = 4 * a.KS;
  // (e4m3 weights come two k-tiles to a 16-byte slot: ranges start and end on even tiles)
  const int ev = W8 ? 1 : 0;
  const int per = ((KC + a.S - 1) / a.S + ev) & ~ev, c_lo = s * per, c_hi = min(KC, c_lo + per);
  const int perw = ((max(c_hi - c_lo, 0) + 3) / 4 + ev) & ~ev, w_lo = c_lo + w * perw,
            w_hi = min(c_hi, w_lo + perw);
  const uint4* wsrc = a.wp + (size_t)nb * (W8 ? KC / 2 : KC) * 64 + lane;
  const uint4* xsrc = a.xp + lane;
  const int lo8 = 2 * c_lo, n8 = 2 * max(c_hi - c_lo, 0);  // this workgroup's k/8 range

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  uint4 bw[2][U], ax[2][U];
  // Loads are unconditional and never touch the loaded data (past the end of the range
  // the weight index is clamped and the activation tile is replaced by a tile of zeros),
  // so the compiler keeps a whole batch in flight behind the MFMAs.  Lanes of rows >=
  // n_rows read the tile of zeros as well (1 KiB that stays in L1): with 8 rows a wave
  // then fetches 256 bytes of operand rows per k-tile from L2 instead of 1 KiB, as much
  // as its weight tile.
  const bool row_lane = (lane & 31) < n_rows;
  auto load = [&](int c, uint4(&b)[U], uint4(&x)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int cc = max(min(c + u, w_hi - 1), 0);
      if constexpr (!W8) b[u] = wsrc[(size_t)cc * 64];
      else if (u < U / 2) b[u] = wsrc[(size_t)max(min((c >> 1) + u, (w_hi >> 1) - 1), 0) * 64];
      if constexpr (XMODE == X_GLOBAL) {
        const uint4* xs = (c + u < w_hi && row_lane) ? xsrc + (size_t)cc * 64 : a.zero_tile + lane;
        x[u] = *xs;
      }
    }
  };
  auto compute = [&](int c, uint4(&b)[U], uint4(&x)[U]) {
    if constexpr (XMODE != X_GLOBAL) {
      const int j = lane & 31, g = lane >> 5;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int cc = max(min(c + u, w_hi - 1), 0);
        x[u] = (j < n_rows && c + u < w_hi) ? xlds[(cc * 2 + g - lo8) * n_rows + j]
                                            : make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (W8) acc = mfma32<F16>(e4m3_slot_half(b[u >> 1], u & 1), x[u], acc);
      else acc = mfma32<F16>(b[u], x[u], acc);
    }
  };

  // Loads return in issue order: row 0, the gains and the first two splits of its partial
  // rows are requested BEFORE the first two batches of weight tiles, which then fly while
  // the row is normalised.
  constexpr int MAXI = XMODE == X_NORM8 ? 8 : 4;  // 4 values per thread and 1024 of the row
  [[maybe_unused]] float4 v[MAXI], gn[MAXI], t0[MAXI], t1[MAXI];
  if constexpr (XMODE != X_GLOBAL) {
    const NormIn& nm = a.norm;
    const size_t pstride = (size_t)nm.part_rows * nm.d;
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
      const int k = tid * 4 + i * 1024;
      v[i] = gn[i] = t0[i] = t1[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k < nm.d) {
        v[i] = *(const float4*)(nm.src + k);
        gn[i] = *(const float4*)(nm.gain + k);
        if (nm.part_S > 0) t0[i] = *(const float4*)(nm.part + k);
        if (nm.part_S > 1) t1[i] = *(const float4*)(nm.part + pstride + k);
      }
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  load(w_lo, bw[0], ax[0]);
  load(w_lo + U, bw[1], ax[1]);
  __builtin_amdgcn_sched_barrier(0);

  if constexpr (XMODE != X_GLOBAL) {
    // RMSNorm of the rows: x * rsqrt(mean(x^2) + eps) * g, with x = source row + partial
    // rows in split order.  One pass over each row: every thread keeps its values in
    // registers, the sum of squares goes through LDS.
    const NormIn& nm = a.norm;
    const int d = nm.d;
    const size_t pstride = (size_t)nm.part_rows * d;
    auto add4 = [](float4& x, const float4& y) { x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w; };
    auto finish_row = [&](int j) {
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        add4(v[i], t0[i]);
        add4(v[i], t1[i]);
      }
      for (int ss = 2; ss < nm.part_S; ++ss) {
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
          const int k = tid * 4 + i * 1024;
          if (k < d) add4(v[i], *(const float4*)(nm.part + ss * pstride + (size_t)j * d + k));
        }
      }
      if (nm.dst && blockIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < MAXI; ++i) {
          const int k = tid * 4 + i * 1024;
          if (k < d) *(float4*)(nm.dst + (size_t)j * nm.dst_stride + k) = v[i];
        }
      }
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < MAXI; ++i)
        ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
      for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
      __syncthreads();  // red is free again
      if (lane == 0) red[0][0][w] = ss;
      __syncthreads();
      const float r =
          rsqrtf((red[0][0][0] + red[0][0][1] + red[0][0][2] + red[0][0][3]) / (float)d + nm.eps);
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const int k = tid * 4 + i * 1024, k8 = k >> 3;
        if (k8 >= lo8 && k8 < lo8 + n8) {  // k >= d: zeros (K padding)
          uint2* dst = (uint2*)&xlds[(k8 - lo8) * n_rows + j];
          dst[(k >> 2) & 1] = make_uint2(pack_op2<F16>(v[i].x * r * gn[i].x, v[i].y * r * gn[i].y),
                                         pack_op2<F16>(v[i].z * r * gn[i].z, v[i].w * r * gn[i].w));
        }
      }
    };
    // row 0 apart from the loop: its loads are older than the weight tiles, and code
    // shared with the later rows would wait for those as well
    finish_row(0);
    for (int j = 1; j < n_rows; ++j) {
#pragma unroll
      for (int i = 0; i < MAXI; ++i) {
        const int k = tid * 4 + i * 1024;
        if (k < d) {
          v[i] = *(const float4*)(nm.src + (size_t)j * nm.src_stride + k);
          if (nm.part_S > 0) t0[i] = *(const float4*)(nm.part + (size_t)j * d + k);
          if (nm.part_S > 1) t1[i] = *(const float4*)(nm.part + pstride + (size_t)j * d + k);
        }
      }
      finish_row(j);
    }
    __syncthreads();
  }

  // The batch a compute phase needs must have been issued BEFORE the batch that flies
  // behind it; the fences stop the instruction scheduler from mixing the phases (which
  // would drain the queue every iteration).
  for (int c = w_lo; c < w_hi; c += 2 * U) {
    compute(c, bw[0], ax[0]);
    __builtin_amdgcn_sched_barrier(0);
    load(c + 2 * U, bw[0], ax[0]);
    __builtin_amdgcn_sched_barrier(0);
    compute(c + U, bw[1], ax[1]);
    __builtin_amdgcn_sched_barrier(0);
    load(c + 3 * U, bw[1], ax[1]);
    __builtin_amdgcn_sched_barrier(0);
  }

  if (w > 0) {
#pragma unroll
    for (int i = 0; i < 16; ++i) red[w - 1][i][lane] = acc[i];
  }
  __syncthreads();
  if (w > 0) return;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] += red[0][i][lane] + red[1][i][lane] + red[2][i][lane];
  if constexpr (W8) scale_tile(a.wscale, nb, lane >> 5, acc);

  if (EPI == EPI_RESID && a.S > 1 && a.e.defer_split) {
    // the split's partial rows [split][row][feature] are left for the consumer (the
    // fused norm of the next projection) to add up: nothing is handed over in here
    const int slot = lane & 31, g = lane >> 5;
    if (slot < n_rows) {
      float* dst = a.e.rpart + ((size_t)s * a.e.rpart_rows + slot) * a.e.d_model + nb * 32 + 4 * g;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *(float4*)(dst + 8 * q4) =
            make_float4(acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2], acc[4 * q4 + 3]);
    }
    return;
  }
  if (a.S > 1) {  // wave 0 alone hands over / collects the partial tile
    float* base = a.partial + (size_t)nb * a.S * 1024;
#pragma unroll
    for (int i = 0; i < 16; ++i) st_coherent(base + (size_t)s * 1024 + i * 64 + lane, acc[i]);
    stores_done();
    int last = 0;
    if (lane == 0) {
      const int old = atomicAdd(a.counters + nb, 1);
      last = (old == a.S - 1);
      if (last) a.counters[nb] = 0;
    }
    last = __shfl(last, 0);
    if (!last) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    for (int ss = 0; ss < a.S; ++ss) {  // fixed order, 16 loads in flight
      float t[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) t[i] = ld_coherent(base + (size_t)ss * 1024 + i * 64 + lane);
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] += t[i];
    }
  }
  const int slot = lane & 31;
  if (slot < n_rows) {
    const int id = (EPI == EPI_LOGITS) ? 0
                   : (a.e.decode_pos >= 0 ? ((slot << 16) | a.e.decode_pos) : a.e.rows[slot]);
    epilogue_tile<EPI, F16>(a.e, nb, slot, id, lane >> 5, acc);
  }
}

template <int MT, int EPI>
static hipError_t set_attr() {
  hipError_t e = hipFuncSetAttribute((const void*)gemm_rows_kernel<MT, EPI, false, false>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 2 * MT * 4096);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute((const void*)gemm_rows_kernel<MT, EPI, true, false>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, 2 * MT * 4096);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute((const void*)gemm_rows_kernel<MT, EPI, true, true>,
                             hipFuncAttributeMaxDynamicSharedMemorySize, 2 * MT * 4096);
}

int gemm_init() {
  hipError_t e;
#define VLAC_SET(MT)                                                    \
  if ((e = set_attr<MT, EPI_QKV>()) != hipSuccess) return (int)e;       \
  if ((e = set_attr<MT, EPI_RESID>()) != hipSuccess) return (int)e;     \
  if ((e = set_attr<MT, EPI_SWIGLU>()) != hipSuccess) return (int)e;    \
  if ((e = set_attr<MT, EPI_LOGITS>()) != hipSuccess) return (int)e;
  VLAC_SET(4)
#undef VLAC_SET
  return gemm_tall_init();
}

template <int MT, bool F16, bool W8>
static void launch_mt(int epi, const GemmArgs& a, int grid, hipStream_t st) {
  const size_t shm = (size_t)2 * MT * 4096;
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_QKV, F16, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_RESID:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_RESID, F16, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_SWIGLU, F16, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_rows_kernel<MT, EPI_LOGITS, F16, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
  }
}

template <bool F16, int XMODE, bool W8>
static void launch_few(int epi, const GemmArgs& a, int grid, size_t shm, hipStream_t st) {
  switch (epi) {
    case EPI_QKV:
      hipLaunchKernelGGL((gemm_few_kernel<EPI_QKV, F16, XMODE, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_RESID:
      hipLaunchKernelGGL((gemm_few_kernel<EPI_RESID, F16, XMODE, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    case EPI_SWIGLU:
      hipLaunchKernelGGL((gemm_few_kernel<EPI_SWIGLU, F16, XMODE, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
    default:
      hipLaunchKernelGGL((gemm_few_kernel<EPI_LOGITS, F16, XMODE, W8>), dim3(grid), dim3(256), shm, st, a);
      break;
  }
}

// LDS budget of the normalised rows (on top of 12 KiB of static LDS)
static const size_t kStageBytes = 49152;

bool gemm_can_fuse_norm(int n_rows_host, int decode_pos, int kpad) {
  return n_rows_host >= 1 && n_rows_host <= 4 && decode_pos >= 0 && kpad <= 8192 &&
         (size_t)(kpad / 8) * n_rows_host * 16 <= kStageBytes;
}

// From this many rows on (the capacity of the launch: streams x tokens; the actual row count
// is known on the device only) the GEMMs go to the kernel built for matrix-core bound
// work.  Measured at the 7B shape, 32 layers, by ACTUAL row count: the one-stream kernel
// wins below about 250 rows (218 rows: 7.1 against 7.8 ms per prefill), the many-rows
// kernel above (327 rows: 10.3 against 9.2 ms, 576 rows: 13.8 against 10.2 ms); a
// capacity of 512 rows (two 7B streams, one stream with two camera views) mostly means
// more than 250 recomputed rows.  (Weights stored as e4m3 codes: the many-rows kernel has
// no variant for them; up to 1023 rows stay with the one-stream kernel, from 1024 rows on
// the matrix is expanded to fp16 before every launch, 3 bytes of traffic per weight
// against the 2 rows flops per weight that such a launch spends on it.)
static const int kTallRows = 512;
// (A launch whose row count is known on the host, a full recompute, goes by that count: from
// kTallKnownRows rows on the many-rows kernel reads the weights once where the one-stream kernel
// fetches them per block of 128 rows: 288 rows of one 7B stream, 32 layers: 8.1 against 9.3 ms;
// 256 rows, two blocks: 7.65 against 7.25 ms, the one-stream kernel keeps them.)
static const int kTallKnownRows = 257;
static bool use_tall(const vlac_ctx* c, int rows_cap, int n_rows_host = -1) {
  if (c->w8) return rows_cap >= 1024 && c->wdeq;
  return rows_cap >= kTallRows || (n_rows_host >= kTallKnownRows && rows_cap > 32);
}

// Most splits the many-rows GEMM with a residual epilogue may use (they need S partial rows
// of fp32 per row in the workspace, and the row kernel that keeps a row in registers)
static int tall_resid_smax(const vlac_ctx* c, int epi, int rows_cap, int d_model) {
  if (epi != EPI_RESID || d_model > 8192) return 1;
  const size_t fit = c->rpart_floats / ((size_t)rows_cap * d_model);
  return fit >= 8 ? 8 : fit >= 3 ? (int)fit : 1;
}

// Split factor of the one-stream kernel (row blocks of 128 rows, MB of them in the grid).
// Split K so that ONE row block (the sparse prefill usually fills one; a full recompute
// runs several side by side) gives about one workgroup per CU.  The projections with
// a residual round up (their splits cost next to nothing: the row kernel that follows
// adds the partial rows); the others round DOWN: their split-K hand-over at the end of
// the kernel costs more than leaving a third of the CUs without a workgroup (measured
// at the 7B shape, 109 rows: gate/up with 172 tiles 52 us unsplit against 63 us in two
// splits; QKV with 96 tiles 42 us in two splits against 52 us in three).
static int rows_kernel_splits(const vlac_ctx* c, int epi, int n_blocks, int KS, int MB, int rpart_rows, int d_model) {
  const int tiles = (n_blocks + 3) / 4;
  int S = epi == EPI_RESID ? (256 + tiles - 1) / tiles : 256 / tiles;
  if (S > KS / 4) S = KS / 4;
  if (S > 8) S = 8;
  if (S < 1) S = 1;
  if (epi == EPI_RESID) {
    while (S > 1 && (size_t)S * rpart_rows * d_model > c->rpart_floats) --S;
  } else {
    while (S > 1 && (size_t)tiles * MB * S * 4 * 4 * 16 * 64 > c->partial_floats) --S;
    if (tiles * MB > c->n_counters) S = 1;
  }
  return S;
}

// Where the many-rows kernel serves a capacity at which a sparse prefill usually leaves
// fewer than kSmallRows rows (the count is known on the device only), BOTH kernels are
// launched for a GEMM and each leaves at once if the count is the other's.  Measured at
// the 7B shape, two streams of 288 tokens: 116 rows 5.6 against 7.9 ms per 32-layer
// prefill, 218 rows 7.3 against 7.8 ms, and 0.4 ms more where the many-rows kernel works
// (128 idle launches of 3 us); at 70 % static about 0.38 of the capacity is recomputed,
// so from a capacity of 768 rows on the second launch would mostly be the idle one; and
// where the reuse lists are too short to leave fewer than kSmallRows rows (top-k 100 of two
// camera views), only the many-rows kernel is launched.
static const int kSmallRows = 257;
// (Rows longer than 8192 elements: the row kernel that adds the partial rows up there takes a
// fixed split factor, so the choice between two kernels with different factors is not offered.)
static bool use_both(const vlac_ctx* c, int rows_cap, int n_rows_host) {
  return use_tall(c, rows_cap, n_rows_host) && !c->w8 && n_rows_host < 0 && rows_cap < 768 && c->rows_floor < kSmallRows &&
         c->cfg.d_model <= 8192;
}

SplitAdapt gemm_resid_adapt(vlac_ctx* c, int n_blocks, int kpad, int rows_cap, const int* n_rows, int n_rows_host) {
  SplitAdapt ad = {nullptr, -1, 0, 0, 0, 0, 0};
  if (!use_tall(c, rows_cap, n_rows_host)) return ad;
  const int d_model = n_blocks * 32;
  const bool both = use_both(c, rows_cap, n_rows_host);
  ad.S_tall = tall_resid_smax(c, EPI_RESID, rows_cap, d_model);
  if (ad.S_tall > 1 || both) {
    ad.n_rows = n_rows;
    ad.n_rows_host = n_rows_host;
    ad.n_blocks = n_blocks;
    ad.KS = kpad / 64;
    if (both) {
      ad.small_below = kSmallRows;
      ad.S_small = rows_kernel_splits(c, EPI_RESID, n_blocks, kpad / 64, kSmallRows / 128, rows_cap, d_model);
    }
  }
  return ad;
}

// the one-stream kernel for up to rows_cap rows; sets and returns a.S
static int launch_rows_kernel(vlac_ctx* c, int epi, GemmArgs& a, int rows_cap, const GemmEpi& e, hipStream_t st) {
  constexpr int MT = 4;
  const int tiles = (a.NB + 3) / 4;
  a.MB = (rows_cap + MT * 32 - 1) / (MT * 32);
  a.S = rows_kernel_splits(c, epi, a.NB, a.KS, a.MB, e.rpart_rows, e.d_model);
  a.P = tiles * a.S;
  const int grid = ((a.P + 7) / 8) * 8 * a.MB;
  if (c->w8) launch_mt<MT, true, true>(epi, a, grid, st);
  else if (c->f16) launch_mt<MT, true, false>(epi, a, grid, st);
  else launch_mt<MT, false, false>(epi, a, grid, st);
  return a.S;
}

int launch_gemm(vlac_ctx* c, int epi, const bf16_t* wp, const float* wscale, int n_blocks, int kpad,
                const bf16_t* xp,
                 const int* n_rows, int n_rows_host, int rows_cap, const GemmEpi& e, hipStream_t st,
                 const NormIn* norm) {
  GemmArgs a;
  a.wp = (const uint4*)wp;
  a.wscale = c->w8 ? wscale : nullptr;
  a.xp = (const uint4*)xp;
  a.zero_tile = (const uint4*)c->zero_tile;
  a.NB = n_blocks;
  a.KS = kpad / 64;
  a.n_rows = n_rows;
  a.n_rows_val = n_rows_host;
  a.rows_lo = 0;
  a.rows_hi = 0x7fffffff;
  memset(&a.norm, 0, sizeof(a.norm));
  if (norm) a.norm = *norm;
  a.partial = c->partial;
  a.counters = c->counters;
  a.e = e;
  const int cls = rows_cap <= 32 ? 0 : 1;
  const bool timed = c->prof_kind == epi + 4 * cls && c->prof_n < c->prof_cap;
  if (timed) (void)hipEventRecord(c->prof_start[c->prof_n], st);
  if (cls == 0) {
    // one workgroup per 32-feature block; K is split over workgroups only when there
    // are fewer blocks than CUs, and never below 32 k-tiles (8 per wave) per workgroup
    const int KC = kpad / 16;
    int S = (256 + n_blocks - 1) / n_blocks;
    if (S > KC / 32) S = KC / 32;
    if (S > 8) S = 8;
    if (S < 1 || n_blocks > c->n_counters || (size_t)n_blocks * 8 * 1024 > c->partial_floats) S = 1;
    a.S = S;
    a.MB = 1;
    a.P = n_blocks * S;
    if (norm) {  // only offered when gemm_can_fuse_norm() holds
      // LDS for the normalised rows: this workgroup's share of K, [k/8][row] 16-byte slices
      const int per = ((KC + S - 1) / S + (c->w8 ? 1 : 0)) & ~(c->w8 ? 1 : 0);  // as in the kernel
      const size_t shm = (size_t)(2 * per) * n_rows_host * 16;
      if (norm->d <= 4096) {
        if (c->w8) launch_few<true, X_NORM4, true>(epi, a, a.P, shm, st);
        else if (c->f16) launch_few<true, X_NORM4, false>(epi, a, a.P, shm, st);
        else launch_few<false, X_NORM4, false>(epi, a, a.P, shm, st);
      } else {
        if (c->w8) launch_few<true, X_NORM8, true>(epi, a, a.P, shm, st);
        else if (c->f16) launch_few<true, X_NORM8, false>(epi, a, a.P, shm, st);
        else launch_few<false, X_NORM8, false>(epi, a, a.P, shm, st);
      }
    } else {
      if (c->w8) launch_few<true, X_GLOBAL, true>(epi, a, a.P, 0, st);
      else if (c->f16) launch_few<true, X_GLOBAL, false>(epi, a, a.P, 0, st);
      else launch_few<false, X_GLOBAL, false>(epi, a, a.P, 0, st);
    }
  } else if (use_tall(c, rows_cap, n_rows_host)) {
    int S_small = 0;
    if (use_both(c, rows_cap, n_rows_host)) {
      GemmArgs r = a;
      r.rows_hi = kSmallRows;
      S_small = launch_rows_kernel(c, epi, r, kSmallRows - 1, e, st);
      a.rows_lo = kSmallRows;
    }
    if (c->w8) {
      launch_expand_e4m3(a.wp, (uint4*)c->wdeq, (size_t)n_blocks * 2 * a.KS, st);
      a.wp = (const uint4*)c->wdeq;
    }
    // (the projections with a residual may split K and leave partial rows to the next row kernel)
    launch_gemm_tall(c->f16, epi, a, rows_cap, tall_resid_smax(c, epi, rows_cap, e.d_model), st);
    if (S_small > a.S) a.S = S_small;  // (the caller learns the most splits either kernel may leave)
  } else {
    launch_rows_kernel(c, epi, a, rows_cap, e, st);
  }
  if (timed) {
    (void)hipEventRecord(c->prof_stop[c->prof_n], st);
    (void)hipEventRecord(c->prof_mark[c->prof_n++], st);  // marker after marker: the bracket's own cost
  }
  return a.S;
}
