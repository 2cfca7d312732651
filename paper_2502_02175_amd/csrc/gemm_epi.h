// Shared by the GEMM kernels: launch arguments and the fused epilogues.
#pragma once
#include "common.h"

struct GemmArgs {
  const uint4* wp;    // weights, fragment order, 64 uint4 per tile (e4m3 codes: per two tiles)
  const float* wscale;  // e4m3 weights: scale per output feature (packed row order), else null
  const uint4* xp;    // activations, fragment order
  const uint4* zero_tile;  // 1 KiB of zeros
  NormIn norm;        // fused RMSNorm of the input rows (few-rows kernel only)
  int NB;             // weight row blocks (32 output features each)
  int KS;             // K steps (64 k = 4 tiles each)
  const int* n_rows;  // device: rows in use
  int n_rows_val;     // >= 0: the row count is known on the host, n_rows is not read
  int rows_lo, rows_hi;  // the launch has work only if rows_lo <= row count < rows_hi (two kernels share a GEMM)
  int S, MB, P;       // split-K factor, row blocks, weight tiles * S
  int x_tiles;        // many-rows GEMM: 32-row tiles the activation buffer holds (copies are clamped to it)
  float* partial;
  int* counters;
  GemmEpi e;
};

// e4m3 weights: a lane's 8 codes of one k-tile (two dwords) -> its 8 fp16 operand values.
// The hardware conversion decodes OCP e4m3 (verified code by code); every e4m3 value is an
// fp16 value, so the second conversion is exact.
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <bool HIGH>
__device__ inline uint32_t e4m3_pair_to_f16(uint32_t codes) {
  const f32x2_t v = __builtin_amdgcn_cvt_pk_f32_fp8((int)codes, HIGH);
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(v.x, v.y));
}
__device__ inline uint4 e4m3_tile_to_f16(uint32_t lo, uint32_t hi) {
  return make_uint4(e4m3_pair_to_f16<false>(lo), e4m3_pair_to_f16<true>(lo),
                    e4m3_pair_to_f16<false>(hi), e4m3_pair_to_f16<true>(hi));
}
// k-tile (2 c + half) of a 16-byte slot that holds the codes of two k-tiles
__device__ inline uint4 e4m3_slot_half(const uint4& slot, int half) {
  return half ? e4m3_tile_to_f16(slot.z, slot.w) : e4m3_tile_to_f16(slot.x, slot.y);
}
// the scales of the 16 results a lane holds of weight block nb (features 8 q + 4 g + i)
__device__ inline void scale_tile(const float* wscale, int nb, int g, f32x16& acc) {
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    const float4 s = *(const float4*)(wscale + nb * 32 + 8 * q4 + 4 * g);
    acc[4 * q4] *= s.x; acc[4 * q4 + 1] *= s.y; acc[4 * q4 + 2] *= s.z; acc[4 * q4 + 3] *= s.w;
  }
}

__device__ inline float silu_f(float x) { return x / (1.f + __expf(-x)); }

template <int EPI, bool F16>
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
            make_uint2(pack_op2<F16>(o1[0], o1[1]), pack_op2<F16>(o1[2], o1[3]));
        *(uint2*)(dst + (size_t)(f2 >> 4) * 512 + ((row + (((f2 >> 3) & 1) << 5)) << 3) + (f2 & 7)) =
            make_uint2(pack_op2<F16>(o2[0], o2[1]), pack_op2<F16>(o2[2], o2[3]));
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
        for (int k = 0; k < 4; ++k) dst[(8 * q4 + 4 * g + k) * 8] = f2op<F16>(acc[4 * q4 + k]);
    }
  } else if constexpr (EPI == EPI_RESID) {
    const int hpos = e.h_compact ? 0 : pos;
    const float* rs = e.resid_src + ((size_t)b * e.resid_seq_stride + hpos) * e.d_model + nb * 32 + 4 * g;
    float* hp = e.h + ((size_t)b * e.h_seq_stride + hpos) * e.d_model + nb * 32 + 4 * g;
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
          make_uint2(pack_op2<F16>(o[0], o[1]), pack_op2<F16>(o[2], o[3]));
    }
  } else {  // EPI_LOGITS: slot is the stream
    float* out = e.logits + (size_t)slot * e.logits_stride + nb * 32 + 4 * g;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
      *(float4*)(out + 8 * q4) =
          make_float4(acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2], acc[4 * q4 + 3]);
  }
}

// gemm_tall.hip: the many-rows kernel with both operands through LDS (its plan: common.h).
// The caller has filled every field of `a` except S, MB, P and x_tiles; S_max: most K splits
// (1 unless the projection adds to the residual stream).
void launch_gemm_tall(bool f16, int epi, GemmArgs& a, int rows_cap, int S_max, hipStream_t st);
int gemm_tall_init();  // kernel attribute setup; returns hipError_t
// e4m3 weight codes (n_slots slots of two k-tiles, 64 uint4 each) -> fp16 tiles, fragment order
void launch_expand_e4m3(const uint4* codes, uint4* tiles, size_t n_slots, hipStream_t st);
