// MFMA formulation of the compressed-cache attention read for one block of
// MFMA_TS prefill tokens (v_mfma_f32_16x16x32_f16, fp32 accumulate).
//
// Key side    D[token][col]   = sum_c  code[token][c] * w[c][col]
//             w[c][col] = q[hq][c] * scale_K[group][c]       (hi and lo fp16 parts)
// Value side  D[col][channel] = sum_t  P[col][t] * code[t][channel]
//             P[col][t] = p[hq][t] * scale_V[t][G]           (hi and lo fp16 parts)
// col = 2*hq + part: the query heads of one KV head (GQA) and the two fp16
// parts of the scaled operand share the 16 MFMA columns.
//
// Codes become MFMA operands with one AND per two codes: the b-bit code that
// sits at bit position s of a 16-bit half is, read as an fp16 DENORMAL,
// code * 2^(s-24); gfx950's MFMA honours fp16 denormals, and the 2^s is undone
// in the other operand.  The zero-point, low-rank and sparse terms are added
// outside the MFMA.
#pragma once
#include "gear_internal.h"

namespace gear {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int MFMA_TS = 512;                 // tokens per block
constexpr float MFMA_OUT_SCALE = 1048576.f;  // 2^24 / 16: undoes the denormal and operand scaling

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_bit_cast(half8, make_uint4(a, b, c, d));
}

// Pairs of one 32-bit code word, in operand order.  Pair v holds the codes at
// index (v, v + P/… ) of the low and high 16-bit halves.
//  2 bits: 16 codes, 8 pairs: pair v = codes (v, v+8), bit shift LG2[v]
//  4 bits:  8 codes, 4 pairs: pair v = codes (v, v+4), bit shift LG4[v]
template <int BITS>
struct Codec;
template <>
struct Codec<2> {
  static constexpr int PAIRS = 8;
  __device__ static __forceinline__ void unpack(uint32_t w, uint32_t* v) {
    v[0] = w & 0x00030003u;
    v[1] = w & 0x000C000Cu;
    v[2] = w & 0x00300030u;
    v[3] = w & 0x00C000C0u;
    v[4] = w & 0x03000300u;
    const uint32_t x = w >> 10;
    v[5] = x & 0x00030003u;
    v[6] = x & 0x000C000Cu;
    v[7] = x & 0x00300030u;
  }
  __device__ static __forceinline__ int lg(int v) { return v < 5 ? 2 * v : 2 * (v - 5); }
};
template <>
struct Codec<4> {
  static constexpr int PAIRS = 4;
  __device__ static __forceinline__ void unpack(uint32_t w, uint32_t* v) {
    v[0] = w & 0x000F000Fu;
    v[1] = w & 0x00F000F0u;
    const uint32_t x = w >> 8;
    v[2] = x & 0x000F000Fu;
    v[3] = x & 0x00F000F0u;
  }
  __device__ static __forceinline__ int lg(int v) { return (v & 1) * 4; }
};

// 2^(4 - lg) as a float (operand scale 16 / 2^lg)
__device__ __forceinline__ float opscale(int lg) { return __uint_as_float((uint32_t)(127 + 4 - lg) << 23); }

// Position of Key channel ch inside the B operand of lane group kg = ch/32:
// returns the fp16 index (0..31) within the lane's 4 k-blocks x 8 slots and the
// bit shift of its pair.
template <int BITS>
__device__ __forceinline__ void key_slot(int r /* ch % 32 */, int& idx, int& lg) {
  if (BITS == 2) {
    const int wi = r >> 4, i = r & 15, p = i >> 3, vv = i & 7;
    idx = (wi * 2 + (vv >> 2)) * 8 + (vv & 3) * 2 + p;
    lg = Codec<2>::lg(vv);
  } else {
    const int jb = r >> 3, i = r & 7, p = i >> 2, v = i & 3;
    idx = jb * 8 + v * 2 + p;
    lg = Codec<4>::lg(v);
  }
}
// Position of token t (inside a Value code block) in the A operand of lane
// group kg: kg, fp16 index within the lane's slots, bit shift.
template <int BITS>
__device__ __forceinline__ void val_slot(int t, int& kg, int& idx, int& lg) {
  if (BITS == 2) {  // 64-token block, 16 tokens per word, two MFMAs
    kg = t >> 4;
    const int i = t & 15, p = i >> 3, vv = i & 7;
    idx = (vv >> 2) * 8 + (vv & 3) * 2 + p;
    lg = Codec<2>::lg(vv);
  } else {  // 32-token block, 8 tokens per word, one MFMA
    kg = t >> 3;
    const int i = t & 7, p = i >> 2, v = i & 3;
    idx = v * 2 + p;
    lg = Codec<4>::lg(v);
  }
}

template <int GQ>
struct MfmaSmem {
  float q[GQ][D];
  float sc[GQ][MFMA_TS];      // raw scores, then p
  float o_fin[GQ][D];
  float kbase[GQ][MFMA_TS / 32];
  float qB[GQ][8];
  float wv[GQ][8];
  float pm[4][GQ][4];
  float red[GQ][4];
  float stat[GQ][2];
};

// Key scores of the block's tokens into S.sc (raw: before the 1/sqrt(d) scale,
// without low-rank and sparse terms but including the zero-point term).
// opnd: this wave's operand staging area (>= 16*128 fp16).
template <int BITS, int GQ>
__device__ __forceinline__ void mfma_key_scores(MfmaSmem<GQ>& S, _Float16* opnd, const Dims& dm, const SegView& ks,
                                                int slab, int t_begin, int t_end) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n16 = lane & 15, kg = lane >> 4;
  const int g = dm.g;
  const int ngroups = MFMA_TS / g;  // uniform over waves; groups past t_end are skipped
  for (int gl = wave; gl < ngroups; gl += 4) {
    const int tg0 = t_begin + gl * g;
    const bool gvalid = tg0 < t_end;
    // ---- operand w = q * scale (hi / lo parts), and the zero-point term
    if (gvalid) {
      float base[GQ];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) base[hq] = 0.0f;
#pragma unroll
      for (int rep = 0; rep < 2; ++rep) {
        const int ch = lane + 64 * rep;
        const uint32_t sb = ks.sz[((size_t)slab * ks.ng_cap + tg0 / g) * D + ch];
        const float delta = h2f(sb & 0xFFFFu), mn = h2f(sb >> 16);
        int idx, lg;
        key_slot<BITS>(ch & 31, idx, lg);
        const float os = opscale(lg);
        _Float16* dst = opnd + (ch >> 5) * 32 + idx;
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) {
          const float qv = S.q[hq][ch];
          const float w = qv * delta * os;
          const _Float16 hi = (_Float16)w;
          const _Float16 lo = (_Float16)(w - (float)hi);
          dst[(2 * hq) * D] = hi;
          dst[(2 * hq + 1) * D] = lo;
          base[hq] += qv * mn;
        }
      }
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        const float b = wave_sum(base[hq]);
        if (lane == 0) S.kbase[hq][gl] = b;
      }
    }
    __syncthreads();
    if (gvalid) {
      half8 bop[4];
#pragma unroll
      for (int jb = 0; jb < 4; ++jb) {
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (n16 < 2 * GQ) raw = *reinterpret_cast<const uint4*>(opnd + n16 * D + kg * 32 + jb * 8);
        bop[jb] = __builtin_bit_cast(half8, raw);
      }
      for (int mt = 0; mt < g / 16; ++mt) {
        const int t = tg0 + 16 * mt + n16;
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        if (BITS == 2) {
          uint2 w = make_uint2(0, 0);
          if (t < t_end) w = *reinterpret_cast<const uint2*>(ks.codes + ((size_t)slab * ks.n_cap + t) * 8 + 2 * kg);
          uint32_t v[8];
          Codec<2>::unpack(w.x, v);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(v[0], v[1], v[2], v[3]), bop[0], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(v[4], v[5], v[6], v[7]), bop[1], acc, 0, 0, 0);
          Codec<2>::unpack(w.y, v);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(v[0], v[1], v[2], v[3]), bop[2], acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(v[4], v[5], v[6], v[7]), bop[3], acc, 0, 0, 0);
        } else {
          uint4 w = make_uint4(0, 0, 0, 0);
          if (t < t_end) w = *reinterpret_cast<const uint4*>(ks.codes + ((size_t)slab * ks.n_cap + t) * 16 + 4 * kg);
          const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
          for (int jb = 0; jb < 4; ++jb) {
            uint32_t v[4];
            Codec<4>::unpack(ww[jb], v);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(v[0], v[1], v[2], v[3]), bop[jb], acc, 0, 0, 0);
          }
        }
        // D[token 4*kg + i][col n16]: add the hi and lo columns, keep the even ones
        const int hq = n16 >> 1;
        float4 s4;
        s4.x = acc[0] + __shfl_xor(acc[0], 1, 64);
        s4.y = acc[1] + __shfl_xor(acc[1], 1, 64);
        s4.z = acc[2] + __shfl_xor(acc[2], 1, 64);
        s4.w = acc[3] + __shfl_xor(acc[3], 1, 64);
        if ((n16 & 1) == 0 && hq < GQ) {
          const float kb = S.kbase[hq][gl];
          s4.x = s4.x * MFMA_OUT_SCALE + kb;
          s4.y = s4.y * MFMA_OUT_SCALE + kb;
          s4.z = s4.z * MFMA_OUT_SCALE + kb;
          s4.w = s4.w * MFMA_OUT_SCALE + kb;
          *reinterpret_cast<float4*>(&S.sc[hq][gl * g + 16 * mt + 4 * kg]) = s4;
        }
      }
    }
    __syncthreads();
  }
}

// Value side: o[hq][c] (quantized backbone incl. zero-point) of the block's
// tokens from p in S.sc.  Results: acc_out[j][i] per lane (column n16 of
// N-tile j, rows 4*kg + i), and S.pm[wave][hq][G] = sum_t p_t * zero_V[t][G].
// opnd: this wave's staging area (>= NG*16*TB fp16).
template <int BITS, int GQ>
__device__ __forceinline__ void mfma_value_accum(MfmaSmem<GQ>& S, _Float16* opnd, const Dims& dm, const SegView& vs,
                                                 int slab, int t_begin, int t_end, floatx4 (&acc)[8]) {
  constexpr int TB = (BITS == 2) ? 64 : 32;  // tokens per code block
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n16 = lane & 15, kg = lane >> 4;
  const int g = dm.g, NG = D / g;
  float pmr[GQ][4];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
    for (int G = 0; G < 4; ++G) pmr[hq][G] = 0.0f;
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};

  for (int bl = wave; bl < MFMA_TS / TB; bl += 4) {
    const int tb0 = t_begin + bl * TB;
    const bool bvalid = tb0 < t_end;
    if (bvalid) {
      // ---- operand P = p * scale_V (hi / lo), and the zero-point sums
      for (int pi = lane; pi < TB * NG; pi += 64) {
        const int tl = pi / NG, G = pi - tl * NG;
        const int tok = tb0 + tl;
        const bool tv = tok < t_end;
        const uint32_t sb = tv ? vs.sz[((size_t)slab * vs.n_cap + tok) * NG + G] : 0u;
        const float delta = h2f(sb & 0xFFFFu), mn = h2f(sb >> 16);
        int skg, idx, lg;
        val_slot<BITS>(tl, skg, idx, lg);
        const float os = opscale(lg);
        _Float16* dst = opnd + (size_t)G * 16 * TB + skg * (TB / 4) + idx;
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) {
          const float pv = tv ? S.sc[hq][tok - t_begin] : 0.0f;
          const float w = pv * delta * os;
          const _Float16 hi = (_Float16)w;
          const _Float16 lo = (_Float16)(w - (float)hi);
          dst[(2 * hq) * TB] = hi;
          dst[(2 * hq + 1) * TB] = lo;
#pragma unroll
          for (int GG = 0; GG < 4; ++GG)
            if (GG == G) pmr[hq][GG] += pv * mn;
        }
      }
    }
    __syncthreads();
    if (bvalid) {
      const uint32_t* cw = vs.codes + ((size_t)slab * vs.nblk_cap + tb0 / TB) * 512 + (kg * 16 + n16) * 8;
      const uint4 c0 = *reinterpret_cast<const uint4*>(cw);
      const uint4 c1 = *reinterpret_cast<const uint4*>(cw + 4);
      const uint32_t words[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
      const int tiles_per_G = g / 16;
      for (int G = 0; G < NG; ++G) {
        const _Float16* src = opnd + (size_t)(G * 16 + n16) * TB + kg * (TB / 4);
        half8 pa0, pa1;
        if (n16 < 2 * GQ) {
          pa0 = __builtin_bit_cast(half8, *reinterpret_cast<const uint4*>(src));
          if (BITS == 2) pa1 = __builtin_bit_cast(half8, *reinterpret_cast<const uint4*>(src + 8));
        } else {
          pa0 = __builtin_bit_cast(half8, make_uint4(0, 0, 0, 0));
          pa1 = pa0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if (j / tiles_per_G == G) {
            if (BITS == 2) {
              uint32_t v[8];
              Codec<2>::unpack(words[j], v);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa0, as_half8(v[0], v[1], v[2], v[3]), acc[j], 0, 0, 0);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa1, as_half8(v[4], v[5], v[6], v[7]), acc[j], 0, 0, 0);
            } else {
              uint32_t v[4];
              Codec<4>::unpack(words[j], v);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa0, as_half8(v[0], v[1], v[2], v[3]), acc[j], 0, 0, 0);
            }
          }
        }
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
    for (int G = 0; G < 4; ++G) {
      const float s = wave_sum(pmr[hq][G]);
      if (lane == 0) S.pm[wave][hq][G] = s;
    }
}

}  // namespace gear
