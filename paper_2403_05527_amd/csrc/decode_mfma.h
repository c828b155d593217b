// MFMA formulation of the compressed-cache attention read for one block of
// MFMA_TS prefill tokens (v_mfma_f32_16x16x32_f16, fp32 accumulate).
//
// Key side    D[col][token]   = sum_c  w[col][c] * code[token][c]
//             w[col][c] = q[hq][c] * scale_K[group][c]       (hi and lo fp16 parts)
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
//
// A block is four independent wavefronts: each owns 128 of the block's tokens
// end to end (scores, its own softmax maximum and sum, Value accumulation,
// low-rank and sparse terms) and the four (m, l, o) states are merged once at
// the end, so no wave ever waits at a barrier in the middle of its work.  Each
// wave issues every global load it needs up front (Key codes into registers;
// scale/zero, low-rank rows and its tiles' outlier lists into its own LDS
// region); only the Value codes are requested later, before the softmax.
#pragma once
#include "gear_internal.h"

namespace gear {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int MFMA_TS = 512;                 // tokens per block (128 per wave)
constexpr float MFMA_OUT_SCALE = 1048576.f;  // 2^24 / 16: undoes the denormal and operand scaling

// Returns w through an empty volatile asm: the unpacking that follows stays where it is
// written (inside the group loop, next to its MFMA) instead of being hoisted out of the
// loop for all tiles at once, which would hold every tile's unpacked codes in registers.
__device__ __forceinline__ uint32_t pin_here(uint32_t w) {
  GEAR_PIN_VGPR(w);
  return w;
}

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_bit_cast(half8, make_uint4(a, b, c, d));
}

// Pairs of one 32-bit code word, in operand order.
//  2 bits: 16 codes, 8 pairs: pair v = codes (v, v+8), bit shift lg(v)
//  4 bits:  8 codes, 4 pairs: pair v = codes (v, v+4), bit shift lg(v)
template <int BITS>
struct Codec;
template <>
struct Codec<2> {
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
  __device__ static __forceinline__ void unpack(uint32_t w, uint32_t* v) {
    v[0] = w & 0x000F000Fu;
    v[1] = w & 0x00F000F0u;
    const uint32_t x = w >> 8;
    v[2] = x & 0x000F000Fu;
    v[3] = x & 0x00F000F0u;
  }
  __device__ static __forceinline__ int lg(int v) { return (v & 1) * 4; }
};

// Two fp16 values as one 32-bit word (a in the low half).
__device__ __forceinline__ uint32_t pack_f16x2(_Float16 a, _Float16 b) {
  return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

// 2^(4 - lg) as a float (operand scale 16 / 2^lg)
__device__ __forceinline__ float opscale(int lg) { return __uint_as_float((uint32_t)(127 + 4 - lg) << 23); }

// R consecutive fp16 (R = 2, 4 or 8; p aligned to 2 R bytes) as floats: one LDS read.
template <int R>
__device__ __forceinline__ void lds_row_f16(const uint16_t* p, float* a) {
  static_assert(R == 2 || R == 4 || R == 8, "one 4-, 8- or 16-byte read");
  uint32_t w[R / 2];
  if constexpr (R == 2) {
    w[0] = *reinterpret_cast<const uint32_t*>(p);
  } else if constexpr (R == 4) {
    const uint2 v = *reinterpret_cast<const uint2*>(p);
    w[0] = v.x; w[1] = v.y;
  } else {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  }
#pragma unroll
  for (int i = 0; i < R / 2; ++i) {
    a[2 * i] = h2f(w[i] & 0xFFFFu);
    a[2 * i + 1] = h2f(w[i] >> 16);
  }
}

// N consecutive floats in LDS (N = 1, 2, 4 or 8; p aligned to 4 N bytes, to 16 for N = 8): one access, two for N = 8.
template <int N>
__device__ __forceinline__ void lds_load_f(const float* p, float (&v)[N]) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "a power of two up to 8");
  if constexpr (N == 1) {
    v[0] = p[0];
  } else if constexpr (N == 2) {
    const float2 t = *reinterpret_cast<const float2*>(p);
    v[0] = t.x; v[1] = t.y;
  } else {
#pragma unroll
    for (int i = 0; i < N; i += 4) {
      const float4 t = *reinterpret_cast<const float4*>(p + i);
      v[i] = t.x; v[i + 1] = t.y; v[i + 2] = t.z; v[i + 3] = t.w;
    }
  }
}
template <int N>
__device__ __forceinline__ void lds_store_f(float* p, const float (&v)[N]) {
  static_assert(N == 1 || N == 2 || N == 4 || N == 8, "a power of two up to 8");
  if constexpr (N == 1) {
    p[0] = v[0];
  } else if constexpr (N == 2) {
    *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
  } else {
#pragma unroll
    for (int i = 0; i < N; i += 4) *reinterpret_cast<float4*>(p + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
  }
}

// Position of Key channel ch (r = ch % 32 inside lane group ch / 32) in the B
// operand: fp16 index (0..31) within the lane's 4 k-blocks x 8 slots, and the
// bit shift of its pair.
template <int BITS>
__device__ __forceinline__ void key_slot(int r, int& idx, int& lg) {
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
// Position of token t of a Value code block in the A operand: lane group,
// fp16 index within the lane's slots, bit shift.
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

// ---------------------------------------------------------------------------
// LDS layout of one MFMA block (byte offsets into dynamic shared memory)
// ---------------------------------------------------------------------------
constexpr int WTOK = 128;  // tokens per wave
// The per-wave float arrays keep the GQ query heads of one row (token, channel) next to each other:
// q[c][hq], score / probability [row][hq], output plane [c][hq], so one LDS access serves all
// heads of a row.  The operand columns are padded by 8 entries: columns that are read by
// different lanes of one instruction then start in different banks.
constexpr int KOP = D + 8;      // Key-side operand column (fp16)
__host__ __device__ constexpr int vop(int tb) { return tb + 8; }   // Value-side operand row of a tb-token code block (fp16)
struct MfmaLayout {
  int q, misc;                                 // shared by the four waves
  int bf, bf_v0, bf_cw, bf_vc;                 // B factors: one (K, V) pair for the block, or one per wave (chunks)
  int wave0, wave_stride;                      // per-wave region
  int sc, szv, ak, av, osp, opnd, qb;          // offsets inside a wave region
  int total;
};
template <int GQ>
struct MfmaMisc {
  float wstat[4][GQ][2];   // per wave: m, l
  float wv[4][GQ][8];      // per wave: p^T A_V
  float pm[4][GQ][4];      // per wave: sum_t p_t * zero_V[t][G]
  int rv[4];               // per wave: rank of its Value factors
};
__host__ __device__ inline int up16i(int x) { return (x + 15) & ~15; }
// rk0, rv0: ranks of the prefill segment; rc: largest rank of an appended chunk (0: no chunk
// blocks in the launch).  The four waves of a prefill block read one copy of B_K and B_V at
// bf and bf + bf_v0; wave w of a chunk block keeps its chunk's pair at bf + w * bf_cw (+ bf_vc).
// lds_rows: the rows of A_K / A_V are staged in LDS.  With four or more query heads per KV head
// the LDS of a block decides how many blocks a CU holds, and the rows then stay in registers
// instead (each lane reads the rows it uses) unless a rank in the launch has no one-read row
// (ranks other than 0, 2, 4, 8).
template <int GQ>
__host__ __device__ inline bool mfma_rows_in_lds(bool odd_rank) { return GQ < 4 || odd_rank; }
template <int GQ>
__host__ __device__ inline MfmaLayout mfma_layout(int bits, int g, int rk0, int rv0, int rc, int ppm, bool odd_rank) {
  MfmaLayout L;
  const int TB = bits == 2 ? 64 : 32, lg = g >= 128 ? 7 : g >= 64 ? 6 : 5, NG = D >> lg;   // g is 32, 64 or 128
  const int rk = rk0 > rc ? rk0 : rc, rv = rv0 > rc ? rv0 : rc;
  int o = 0;
  L.q = o; o += GQ * D * 4;
  L.misc = o; o += up16i((int)sizeof(MfmaMisc<GQ>));
  L.bf = o;
  L.bf_v0 = up16i(D * rk0 * 2);
  L.bf_vc = up16i(D * rc * 2);
  L.bf_cw = 2 * L.bf_vc;
  {
    const int shared = L.bf_v0 + up16i(D * rv0 * 2), per_wave = 4 * L.bf_cw;
    o += shared > per_wave ? shared : per_wave;
  }
  L.wave0 = o;
  int w = 0;
  L.sc = w; w += GQ * WTOK * 4;
  L.szv = w; w += WTOK * NG * 4;
  L.ak = w; w += mfma_rows_in_lds<GQ>(odd_rank) ? up16i(WTOK * rk * 2) : 0;
  L.av = w; w += mfma_rows_in_lds<GQ>(odd_rank) ? up16i(WTOK * rv * 2) : 0;
  int oh = 2 * GQ * KOP;
  if (NG * 2 * GQ * vop(TB) > oh) oh = NG * 2 * GQ * vop(TB);
  L.opnd = w; w += oh * 2;
  L.osp = L.opnd;   // the output plane (GQ * 128 floats <= the operand area) is written after the last operand was read
  L.qb = w; w += GQ * 8 * 4;
  L.wave_stride = up16i(w);
  L.total = L.wave0 + 4 * L.wave_stride;
  return L;
}

// q^T B_K for a rank whose row of B_K is one LDS read (R = 2, 4 or 8), added into SqB[hq * 8 + r]
// (zero on entry).  Up to four query heads per pass, 64 / heads lanes each (whole rows of 16 lanes):
// a lane sums its share of the 128 channels for all R ranks at once, the rows of 16 reduce R values
// together, and the rows of one head meet in an LDS add (in a fixed lane order: the sum does not
// vary from run to run).
template <int GQ, int R>
__device__ __forceinline__ void query_down_projection(const float* Sq, const uint16_t* Sbf, float* SqB, int lane) {
  constexpr int HP = GQ < 4 ? GQ : 4;   // query heads per pass
  constexpr int LPH = 64 / HP;          // lanes per head
  constexpr int CPL = D / LPH;          // channels per lane
  const int hl = lane / LPH, part = lane % LPH;
#pragma unroll
  for (int h0 = 0; h0 < GQ; h0 += HP) {
    const int hq = h0 + hl;
    float s[R];
#pragma unroll
    for (int r = 0; r < R; ++r) s[r] = 0.0f;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = part + LPH * i;     // the lanes of a head read consecutive channels
      const float qv = Sq[c * GQ + hq];
      float b[R];
      lds_row_f16<R>(Sbf + c * R, b);
#pragma unroll
      for (int r = 0; r < R; ++r) s[r] += qv * b[r];
    }
    if constexpr (R == 2) {
      const float u = row16_sum2(s[0], s[1], lane);
      if ((lane & 15) < 2) atomicAdd(&SqB[hq * 8 + (lane & 1)], u);
    } else {
      const float u = row16_sum4(s[0], s[1], s[2], s[3], lane);
      if ((lane & 15) < 4) atomicAdd(&SqB[hq * 8 + (lane & 3)], u);
      if constexpr (R == 8) {
        const float u2 = row16_sum4(s[4], s[5], s[6], s[7], lane);
        if ((lane & 15) < 4) atomicAdd(&SqB[hq * 8 + 4 + (lane & 3)], u2);
      }
    }
  }
}

// Low-rank Key term of the rows lane and lane + 64 (their scores sc[rep][hq] are in registers) for a
// rank that is one LDS read per row: score[row] += A_K[row] . (q^T B_K).
// (REGS: the two rows as loaded by the lane itself; otherwise they are read from LDS)
template <int R>
__device__ __forceinline__ void reg_row_f16(const uint4& v, float* a) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < R / 2; ++i) {
    a[2 * i] = h2f(w[i] & 0xFFFFu);
    a[2 * i + 1] = h2f(w[i] >> 16);
  }
}
template <int GQ, int R, bool REGS>
__device__ __forceinline__ void lowrank_key_rows(const uint16_t* Sak, const uint4 (&regs)[2], const float* SqB,
                                                 float (&sc)[2][GQ], int lane, int nw) {
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) {
    const int row = lane + 64 * rep;
    if (row < nw) {
      float a[R];
      if constexpr (REGS) reg_row_f16<R>(regs[rep], a);
      else lds_row_f16<R>(Sak + row * R, a);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        float s = sc[rep][hq];
#pragma unroll
        for (int r = 0; r < R; ++r) s += SqB[hq * 8 + r] * a[r];
        sc[rep][hq] = s;
      }
    }
  }
}
// p^T A_V over the wave's rows (probabilities pr[rep][hq] of rows lane, lane + 64 in registers) for such a
// rank, added into wv[hq * 8 + r] (zero on entry).
template <int GQ, int R, bool REGS>
__device__ __forceinline__ void lowrank_value_down(const uint16_t* Sav, const uint4 (&regs)[2], const float (&pr)[2][GQ],
                                                   float* wv, int lane, int nw) {
  float part[GQ][R];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
    for (int r = 0; r < R; ++r) part[hq][r] = 0.0f;
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) {
    const int row = lane + 64 * rep;
    if (row < nw) {
      float a[R];
      if constexpr (REGS) reg_row_f16<R>(regs[rep], a);
      else lds_row_f16<R>(Sav + row * R, a);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        const float p = pr[rep][hq];
#pragma unroll
        for (int r = 0; r < R; ++r) part[hq][r] += p * a[r];
      }
    }
  }
  // the four rows of 16 lanes add their sums into LDS (fixed lane order inside the one instruction)
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    if constexpr (R == 2) {
      const float u = row16_sum2(part[hq][0], part[hq][1], lane);
      if ((lane & 15) < 2) atomicAdd(&wv[hq * 8 + (lane & 1)], u);
    } else {
#pragma unroll
      for (int r0 = 0; r0 < R; r0 += 4) {
        const float u = row16_sum4(part[hq][r0], part[hq][r0 + 1], part[hq][r0 + 2], part[hq][r0 + 3], lane);
        if ((lane & 15) < 4) atomicAdd(&wv[hq * 8 + r0 + (lane & 3)], u);
      }
    }
  }
}

// Row `row` of a rank-rk factor (rk = 2, 4 or 8; 2 rk bytes) from a view of the wave's rows; 0 past the view.
__device__ __forceinline__ uint4 load_factor_row(GEAR_BUF_T view, int row, int rk) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (rk == 8) {
    v = GEAR_BUF_LOAD16(view, row * 16);
  } else if (rk == 4) {
    const uint2 t = GEAR_BUF_LOAD8(view, row * 8);
    v.x = t.x; v.y = t.y;
  } else if (rk == 2) {
    v.x = GEAR_BUF_LOAD4(view, row * 4);
  }
  return v;
}

// One block: each of the four waves takes up to 128 consecutive token rows [tw0, tw0 + nw)
// of the stored segment it is given (ks, vs may differ from wave to wave: the prefill
// segment for every wave, or one appended chunk per wave), all of slab (b, h).  Writes
// the block's merged partial softmax record (m, l, o[128]) of each of the GQ query
// heads.  rk0 / rv0 / rc size the LDS layout (see mfma_layout); shared_b: the four waves
// read the same segment (a prefill block), so its B factors are staged once.
template <int BITS, int GQ, int LG>
__device__ void mfma_block(unsigned char* smem, const Dims& dm, const SegView& ks, const SegView& vs,
                           const uint16_t* __restrict__ qg /* q of query head h*GQ of batch b */, int slab, int b,
                           int tw0, int nw, int rk0, int rv0, int rc, bool odd_rank, bool shared_b,
                           float* __restrict__ rec_base, int rec_stride) {
  constexpr int TB = (BITS == 2) ? 64 : 32;   // tokens per Value code block
  constexpr int KW = (BITS == 2) ? 2 : 4;     // Key code words per lane per M-tile
  constexpr int VBLK = WTOK / TB;             // Value blocks per wave
  const int tid = threadIdx.x, wave = GEAR_WAVE_UNIFORM(tid >> 6), lane = tid & 63;
  const int n16 = lane & 15, kg = lane >> 4;
  constexpr int g = 1 << LG, lg = LG, NG = D >> LG;   // the group size (32, 64 or 128) is a template parameter: group loops unroll
  const int rk = ks.rank, rv = vs.rank;
  const MfmaLayout L = mfma_layout<GQ>(BITS, g, rk0, rv0, rc, dm.ppm, odd_rank);
  const bool rows_lds = mfma_rows_in_lds<GQ>(odd_rank);   // compile-time true for fewer than four query heads
  float* Sq = reinterpret_cast<float*>(smem + L.q);                 // [128][GQ]
  MfmaMisc<GQ>& M = *reinterpret_cast<MfmaMisc<GQ>*>(smem + L.misc);
  unsigned char* wbase = smem + L.wave0 + (size_t)wave * L.wave_stride;
  float* Ssc = reinterpret_cast<float*>(wbase + L.sc);              // [128][GQ] raw scores, then p
  uint32_t* Sszv = reinterpret_cast<uint32_t*>(wbase + L.szv);      // [128][NG]
  uint16_t* Sak = reinterpret_cast<uint16_t*>(wbase + L.ak);        // [128][rk]
  uint16_t* Sav = reinterpret_cast<uint16_t*>(wbase + L.av);
  uint16_t* Sbfk = reinterpret_cast<uint16_t*>(smem + L.bf + (shared_b ? 0 : wave * L.bf_cw));   // [128][rk]
  uint16_t* Sbfv = reinterpret_cast<uint16_t*>(smem + L.bf + (shared_b ? L.bf_v0 : wave * L.bf_cw + L.bf_vc));
  float* Sosp = reinterpret_cast<float*>(wbase + L.osp);            // [128][GQ] this wave's output plane (shares the operand area)
  _Float16* opnd = reinterpret_cast<_Float16*>(wbase + L.opnd);
  float* SqB = reinterpret_cast<float*>(wbase + L.qb);              // [GQ][8] q^T B_K
  const float scale = 0.08838834764831845f;  // 1/sqrt(128)
  nw = GEAR_WAVE_UNIFORM(nw < 0 ? 0 : (nw > WTOK ? WTOK : nw));   // rows this wave owns (may be 0)
  tw0 = GEAR_WAVE_UNIFORM(tw0);

  // =================== prologue: every load in flight ===================
  // the (offset, count) entries of this wave's two tiles of each tensor
  uint2 tab = make_uint2(0, 0);
  if (dm.ppm > 0 && lane < 4) {
    const int ti = lane & 1;
    if (ti * TILE < nw) {
      const int tile = tw0 / TILE + ti;
      tab = (lane < 2) ? ks.sp_table[(size_t)slab * ks.ntile_cap + tile] : vs.sp_table[(size_t)slab * vs.ntile_cap + tile];
    }
  }
  // Key codes of this wave's 8 M-tiles into registers (rows past the wave's last read as 0)
  uint32_t kw[8][KW];
  {
    constexpr int ROWB = 16 * BITS;   // bytes of one token's codes
    const GEAR_BUF_T kbuf = GEAR_BUF_MAKE(ks.codes + ((size_t)slab * ks.n_cap + tw0) * (4 * BITS), nw * ROWB);
    const uint32_t koff = n16 * ROWB + kg * (KW * 4);
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      if constexpr (BITS == 2) {
        const uint2 w = GEAR_BUF_LOAD8(kbuf, koff + mt * 16 * ROWB);
        kw[mt][0] = w.x; kw[mt][1] = w.y;
      } else {
        const uint4 w = GEAR_BUF_LOAD16(kbuf, koff + mt * 16 * ROWB);
        kw[mt][0] = w.x; kw[mt][1] = w.y; kw[mt][2] = w.z; kw[mt][3] = w.w;
      }
    }
  }
  // shared q and B factors, this wave's (scale, zero) and rows of A: first every load
  // into registers (16 bytes per lane and request), LDS writes afterwards, so that all
  // of them are in flight together.  The arena keeps these arrays 16-byte aligned per
  // slab and padded, so whole 16-byte pieces may be read past the wave's last row.
  uint32_t qreg[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int i = tid + 256 * k;
    qreg[k] = 0u;
    if (i < GQ * D / 2) qreg[k] = reinterpret_cast<const uint32_t*>(qg)[i];
  }
  const int ngl = (nw + g - 1) >> lg;
  const int n4_szk = ngl * (D / 4), n4_szv = (nw * NG + 3) >> 2, n4_ak = rows_lds ? (nw * rk + 7) >> 3 : 0,
            n4_av = rows_lds ? (nw * rv + 7) >> 3 : 0;
  const bool stage_b = shared_b ? wave == 0 : nw > 0;   // a prefill block's first wave always owns rows
  const int n4_bk = stage_b ? 16 * rk : 0, n4_bv = stage_b ? 16 * rv : 0;   // 128 * rank fp16
  // (per-vector grouping: a segment's one Key group, and the wave's 128 rows lie in it)
  const uint32_t* g_szk = reinterpret_cast<const uint32_t*>(ks.sz + ((size_t)slab * ks.ng_cap + (dm.kcvt ? 0 : tw0 >> lg)) * D);
  const uint4* g_szv = reinterpret_cast<const uint4*>(vs.sz + ((size_t)slab * vs.n_cap + tw0) * NG);
  const uint4* g_ak = reinterpret_cast<const uint4*>(ks.A + ((size_t)slab * ks.n_cap + tw0) * rk);
  const uint4* g_av = reinterpret_cast<const uint4*>(vs.A + ((size_t)slab * vs.n_cap + tw0) * rv);
  const uint4* g_bk = reinterpret_cast<const uint4*>(ks.Bf + (size_t)slab * D * rk);
  const uint4* g_bv = reinterpret_cast<const uint4*>(vs.Bf + (size_t)slab * D * rv);
  // piece lane of each array; pieces 64.. (g = 32, rank 8) follow after the first
  // The lane builds the Key operand of two channels whose fp16 halves share a 32-bit word of the operand
  // column (key_slot: channels PD apart inside a block of 2 PD), so every operand store is a whole word.
  constexpr int PD = (BITS == 2) ? 8 : 4;
  const int kc0 = (lane / PD) * (2 * PD) + (lane % PD);   // the lane's channels: kc0 and kc0 + PD
  // their (scale, zero) in each of the wave's groups: straight into registers
  uint32_t szk_r[WTOK >> LG][2];
  {
    const GEAR_BUF_T zbuf = GEAR_BUF_MAKE(g_szk, n4_szk * 16);   // groups past the wave's last row read as 0
#pragma unroll
    for (int gw = 0; gw < (WTOK >> LG); ++gw)
#pragma unroll
      for (int rep = 0; rep < 2; ++rep) szk_r[gw][rep] = GEAR_BUF_LOAD4(zbuf, (gw * D + kc0 + PD * rep) * 4);
  }
  const uint4 r_szv = GEAR_BUF_LOAD16(GEAR_BUF_MAKE(g_szv, n4_szv * 16), lane * 16);
  const uint4 r_ak = GEAR_BUF_LOAD16(GEAR_BUF_MAKE(g_ak, n4_ak * 16), lane * 16);
  const uint4 r_av = GEAR_BUF_LOAD16(GEAR_BUF_MAKE(g_av, n4_av * 16), lane * 16);
  const uint4 r_bk = GEAR_BUF_LOAD16(GEAR_BUF_MAKE(g_bk, n4_bk * 16), lane * 16);
  const uint4 r_bv = GEAR_BUF_LOAD16(GEAR_BUF_MAKE(g_bv, n4_bv * 16), lane * 16);
  uint4 akr[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};   // rows lane, lane + 64 of A_K when they are not staged
  if (!rows_lds) {
    const GEAR_BUF_T av = GEAR_BUF_MAKE(g_ak, nw * rk * 2);
    akr[0] = load_factor_row(av, lane, rk);
    akr[1] = load_factor_row(av, lane + 64, rk);
  }
  // outlier lists of the wave's tiles: K tiles then V tiles, rows rebased to the wave
  // a table entry is trusted only as far as its pool reaches
  {
    const uint32_t cap = (lane < 2) ? ks.pool_cap : vs.pool_cap;
    if (tab.x > cap) tab.x = cap;
    if (tab.y > cap - tab.x) tab.y = cap - tab.x;
  }
  const uint32_t ck0 = __shfl(tab.y, 0, 64), ck1 = __shfl(tab.y, 1, 64);
  const uint32_t cv0 = __shfl(tab.y, 2, 64), cv1 = __shfl(tab.y, 3, 64);
  const uint32_t ok0 = __shfl(tab.x, 0, 64), ok1 = __shfl(tab.x, 1, 64);
  const uint32_t ov0 = __shfl(tab.x, 2, 64), ov1 = __shfl(tab.x, 3, 64);
  const uint32_t* poolk = ks.sp_pool + (size_t)slab * ks.pool_cap;
  const uint32_t* poolv = vs.sp_pool + (size_t)b * vs.pool_cap;
  // overflow lists: the first SPR * 64 entries travel in registers, entry lane + 64 i,
  // as (row in the wave) * 128 + c | value << 16
  constexpr int SPR = 1;
  uint32_t spk_r[SPR], spv_r[SPR];
#pragma unroll
  for (int i = 0; i < SPR; ++i) {
    const uint32_t e = lane + 64 * i;
    spk_r[i] = 0u;
    spv_r[i] = 0u;
    if (e < ck0 + ck1) {
      const bool second = e >= ck0;
      const uint32_t en = second ? poolk[ok1 + (e - ck0)] : poolk[ok0 + e];
      spk_r[i] = en + (second ? TILE * D : 0);
    }
    if (e < cv0 + cv1) {
      const bool second = e >= cv0;
      const uint32_t en = second ? poolv[ov1 + (e - cv0)] : poolv[ov0 + e];
      spv_r[i] = en + (second ? TILE * D : 0);
    }
  }
  // everything is requested; now the LDS writes
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int i = tid + 256 * k;
    if (i < GQ * D / 2) {   // channels c, c + 1 of query head hq
      const int hq = i / (D / 2), c = 2 * (i % (D / 2));
      Sq[c * GQ + hq] = h2f(qreg[k] & 0xFFFFu);
      Sq[(c + 1) * GQ + hq] = h2f(qreg[k] >> 16);
    }
  }
  if (lane < n4_szv) reinterpret_cast<uint4*>(Sszv)[lane] = r_szv;
  if (lane < n4_ak) reinterpret_cast<uint4*>(Sak)[lane] = r_ak;
  if (lane < n4_av) reinterpret_cast<uint4*>(Sav)[lane] = r_av;
  if (lane < n4_bk) reinterpret_cast<uint4*>(Sbfk)[lane] = r_bk;
  if (lane < n4_bv) reinterpret_cast<uint4*>(Sbfv)[lane] = r_bv;
  if (n4_szv > 64 || n4_ak > 64 || n4_av > 64 || n4_bk > 64 || n4_bv > 64) {   // wave-uniform: second pieces
    const int j = lane + 64;
    if (j < n4_szv) reinterpret_cast<uint4*>(Sszv)[j] = g_szv[j];
    if (j < n4_ak) reinterpret_cast<uint4*>(Sak)[j] = g_ak[j];
    if (j < n4_av) reinterpret_cast<uint4*>(Sav)[j] = g_av[j];
    if (j < n4_bk) reinterpret_cast<uint4*>(Sbfk)[j] = g_bk[j];
    if (j < n4_bv) reinterpret_cast<uint4*>(Sbfv)[j] = g_bv[j];
  }
  if (lane < GQ * 8) (&M.wv[wave][0][0])[lane] = 0.0f;
  if (lane < GQ * 4) (&M.pm[wave][0][0])[lane] = 0.0f;
  block_lds_sync();   // q and the B factors are visible to all waves; from here on waves run independently

  // fixed outlier slots of the Key rows lane and lane + 64 (an empty slot is 0: channel 0,
  // value +0); they arrive while the Key scores are computed
  uint4 ellk[2];
  {
    static_assert(ELL_K == 4, "one 16-byte read per row");
    const GEAR_BUF_T ebuf = GEAR_BUF_MAKE(ks.ell + ((size_t)slab * ks.n_cap + tw0) * ELL_K, dm.ppm > 0 ? nw * 16 : 0);
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) ellk[rep] = GEAR_BUF_LOAD16(ebuf, (lane + 64 * rep) * 16);
  }

  // q^T B_K (down-projection of the low-rank Key term) into SqB[hq][r]
  if (rk > 0) {
    for (int i = lane; i < GQ * 8; i += 64) SqB[i] = 0.0f;   // slots r >= rk stay 0
    wave_lds_sync();
    if (rk == 4) query_down_projection<GQ, 4>(Sq, Sbfk, SqB, lane);
    else if (rk == 2) query_down_projection<GQ, 2>(Sq, Sbfk, SqB, lane);
    else if (rk == 8) query_down_projection<GQ, 8>(Sq, Sbfk, SqB, lane);
    else {
      // any other rank: the GQ * rkp outputs (rkp = rank rounded up to a power of two) are spread over
      // the 64 lanes, P lanes per output, each summing 128 / P channels; a butterfly over the P lanes
      // finishes the sums
      const int lrk = rk <= 1 ? 0 : rk <= 2 ? 1 : rk <= 4 ? 2 : 3, rkp = 1 << lrk;
      constexpr int LGQ = GQ == 1 ? 0 : GQ == 2 ? 1 : GQ == 4 ? 2 : 3;
      const int lP = 6 - LGQ - lrk, P = 1 << lP;   // 64 / (GQ * rkp)
      const int outi = lane >> lP, part = lane & (P - 1);
      const int hq = outi >> lrk, r = outi & (rkp - 1);
      float s = 0.0f;
      if (r < rk)
        for (int c = part; c < D; c += P) s += Sq[c * GQ + hq] * h2f(Sbfk[c * rk + r]);
      for (int o = 1; o < P; o <<= 1) s += __shfl_xor(s, o, 64);
      if (part == 0) SqB[hq * 8 + r] = s;
    }
    wave_lds_sync();
  }

  // =================== Key scores on the matrix cores ===================
  int kslot0;       // operand position of channel kc0 (even; kc0 + PD follows it; the same for every group)
  float kscale;
  {
    int idx, lg;
    key_slot<BITS>(kc0 & 31, idx, lg);
    kslot0 = (kc0 >> 5) * 32 + idx;
    kscale = opscale(lg);
  }
#pragma unroll
  for (int gw = 0; gw < (WTOK >> lg); ++gw) {
    if (gw * g >= nw) break;                        // wave-uniform
    float kb[GQ];
    uint32_t first[GQ];   // (hi, lo) parts of the first channel's operand
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) kb[hq] = 0.0f;
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      const int ch = kc0 + PD * rep;
      const uint32_t sb = szk_r[gw][rep];
      const float delta = h2f(sb & 0xFFFFu), mn = h2f(sb >> 16);
      float qh[GQ];
      lds_load_f<GQ>(Sq + ch * GQ, qh);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        const float qv = qh[hq];
        const float w = qv * delta * kscale;
        const _Float16 hi = (_Float16)w;
        const _Float16 lo = (_Float16)(w - (float)hi);
        kb[hq] += qv * mn;
        if (rep == 0) {
          first[hq] = pack_f16x2(hi, lo);
        } else {
          const uint32_t second = pack_f16x2(hi, lo);
          *reinterpret_cast<uint32_t*>(opnd + (2 * hq) * KOP + kslot0) = GEAR_BYTE_PERM(second, first[hq], 0x05040100u);
          *reinterpret_cast<uint32_t*>(opnd + (2 * hq + 1) * KOP + kslot0) = GEAR_BYTE_PERM(second, first[hq], 0x07060302u);
        }
      }
    }
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) kb[hq] = wave_sum(kb[hq]);   // zero-point term q . zero_K of the group
    wave_lds_sync();
    half8 bop[4];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (n16 < 2 * GQ) raw = *reinterpret_cast<const uint4*>(opnd + n16 * KOP + kg * 32 + jb * 8);
      bop[jb] = __builtin_bit_cast(half8, raw);
    }
    // lane group kg receives columns 4 kg .. 4 kg + 3: both parts of query heads 2 kg and 2 kg + 1
    const int hq0 = 2 * kg, hq1 = 2 * kg + 1;
    float kb0 = 0.0f, kb1 = 0.0f;
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      kb0 = (hq == hq0) ? kb[hq] : kb0;
      kb1 = (hq == hq1) ? kb[hq] : kb1;
    }
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
      if ((mt >> (lg - 4)) == gw) {   // tile mt (16 tokens) lies in group gw
        floatx4 acc = {0.f, 0.f, 0.f, 0.f};
        if (BITS == 2) {
          uint32_t v[8];
          Codec<2>::unpack(pin_here(kw[mt][0]), v);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(bop[0], as_half8(v[0], v[1], v[2], v[3]), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(bop[1], as_half8(v[4], v[5], v[6], v[7]), acc, 0, 0, 0);
          Codec<2>::unpack(pin_here(kw[mt][1]), v);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(bop[2], as_half8(v[0], v[1], v[2], v[3]), acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(bop[3], as_half8(v[4], v[5], v[6], v[7]), acc, 0, 0, 0);
        } else {
#pragma unroll
          for (int jb = 0; jb < 4; ++jb) {
            uint32_t v[4];
            Codec<4>::unpack(pin_here(kw[mt][jb % KW]), v);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(bop[jb], as_half8(v[0], v[1], v[2], v[3]), acc, 0, 0, 0);
          }
        }
        // D[col 4*kg + i][token n16]: the hi and lo columns of a query head sit in one lane
        const float s0 = (acc[0] + acc[1]) * MFMA_OUT_SCALE + kb0, s1 = (acc[2] + acc[3]) * MFMA_OUT_SCALE + kb1;
        if constexpr (GQ == 1) {
          if (kg == 0) Ssc[16 * mt + n16] = s0;
        } else {
          if (hq0 < GQ) *reinterpret_cast<float2*>(&Ssc[(16 * mt + n16) * GQ + hq0]) = make_float2(s0, s1);
        }
      }
    }
    wave_lds_sync();
  }

  // Sparse Key term, overflow entries (rows with more outliers than fixed slots): LDS float adds
  // into the stored scores; those of one wave are applied in program order and in a fixed lane
  // order inside one instruction, so the result does not vary from run to run.
  if (dm.ppm > 0 && ck0 + ck1 > 0) {   // wave-uniform
    auto add_k = [&](uint32_t en) {
      const int row = (en & 0xFFFFu) >> 7, c = en & 127u;
      const float v = h2f(en >> 16);
      float qh[GQ];
      lds_load_f<GQ>(Sq + c * GQ, qh);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) atomicAdd(&Ssc[row * GQ + hq], qh[hq] * v);
    };
#pragma unroll
    for (int i = 0; i < SPR; ++i)
      if ((uint32_t)(lane + 64 * i) < ck0 + ck1) add_k(spk_r[i]);
    for (uint32_t e = SPR * 64 + lane; e < ck0 + ck1; e += 64) {   // longer lists: the rest from global memory
      const bool second = e >= ck0;
      const uint32_t en = second ? poolk[ok1 + (e - ck0)] : poolk[ok0 + e];
      add_k(en + (second ? TILE * D : 0));
    }
    wave_lds_sync();
  }

  // From here the lane owns rows lane and lane + 64: their scores of all query heads stay in
  // registers through the low-rank term, the fixed outlier slots and the softmax.
  float sc[2][GQ];
#pragma unroll
  for (int rep = 0; rep < 2; ++rep) lds_load_f<GQ>(Ssc + (lane + 64 * rep) * GQ, sc[rep]);   // rows >= nw: masked below

  // low-rank Key term
  if (rk == 4) {
    if (rows_lds) lowrank_key_rows<GQ, 4, false>(Sak, akr, SqB, sc, lane, nw);
    else lowrank_key_rows<GQ, 4, true>(Sak, akr, SqB, sc, lane, nw);
  } else if (rk == 2) {
    if (rows_lds) lowrank_key_rows<GQ, 2, false>(Sak, akr, SqB, sc, lane, nw);
    else lowrank_key_rows<GQ, 2, true>(Sak, akr, SqB, sc, lane, nw);
  } else if (rk == 8) {
    if (rows_lds) lowrank_key_rows<GQ, 8, false>(Sak, akr, SqB, sc, lane, nw);
    else lowrank_key_rows<GQ, 8, true>(Sak, akr, SqB, sc, lane, nw);
  } else if (rk > 0) {
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      const int row = lane + 64 * rep;
      float a[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) a[r] = (r < rk && row < nw) ? h2f(Sak[row * rk + r]) : 0.0f;
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        const float4 b0 = *reinterpret_cast<const float4*>(&SqB[hq * 8]);       // entries r >= rk are unused (a = 0)
        const float4 b1 = *reinterpret_cast<const float4*>(&SqB[hq * 8 + 4]);
        float s = sc[rep][hq];
        s += b0.x * a[0] + b0.y * a[1] + b0.z * a[2] + b0.w * a[3];
        if (rk > 4) s += b1.x * a[4] + b1.y * a[5] + b1.z * a[6] + b1.w * a[7];
        sc[rep][hq] = s;
      }
    }
  }

  // sparse Key term, fixed slots of the lane's own rows
  if (dm.ppm > 0) {
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      const uint32_t es[4] = {ellk[rep].x, ellk[rep].y, ellk[rep].z, ellk[rep].w};
      float a2[GQ];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) a2[hq] = 0.0f;
#pragma unroll
      for (int i = 0; i < ELL_K; ++i) {
        const float v = h2f(es[i] >> 16);
        const int c = es[i] & 127u;
        float qh[GQ];
        lds_load_f<GQ>(Sq + c * GQ, qh);
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) a2[hq] += qh[hq] * v;
      }
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) sc[rep][hq] += a2[hq];
    }
  }

  uint4 avr[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};   // rows lane, lane + 64 of A_V when they are not staged
  if (!rows_lds) {
    const GEAR_BUF_T av = GEAR_BUF_MAKE(g_av, nw * rv * 2);
    avr[0] = load_factor_row(av, lane, rv);
    avr[1] = load_factor_row(av, lane + 64, rv);
  }
  // request this wave's Value codes; they arrive while the softmax runs
  uint32_t vw[VBLK][8];
#pragma unroll
  for (int bl = 0; bl < VBLK; ++bl) {
    const int tb0 = tw0 + bl * TB;
#pragma unroll
    for (int j = 0; j < 8; ++j) vw[bl][j] = 0u;
    if (bl * TB < nw) {
      const uint32_t* cw = vs.codes + ((size_t)slab * vs.nblk_cap + tb0 / TB) * 512 + (kg * 16 + n16) * 8;
      const uint4 c0 = *reinterpret_cast<const uint4*>(cw);
      const uint4 c1 = *reinterpret_cast<const uint4*>(cw + 4);
      vw[bl][0] = c0.x; vw[bl][1] = c0.y; vw[bl][2] = c0.z; vw[bl][3] = c0.w;
      vw[bl][4] = c1.x; vw[bl][5] = c1.y; vw[bl][6] = c1.z; vw[bl][7] = c1.w;
    }
  }

  // =================== this wave's softmax state ===================
  float pr[2][GQ];   // probabilities of rows lane, lane + 64 (0 for rows >= nw)
  {
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      const float s0 = lane < nw ? sc[0][hq] * scale : -INFINITY;
      const float s1 = lane + 64 < nw ? sc[1][hq] * scale : -INFINITY;
      const float m = wave_max(fmaxf(s0, s1));
      const float p0 = lane < nw ? __expf(s0 - m) : 0.0f;
      const float p1 = lane + 64 < nw ? __expf(s1 - m) : 0.0f;
      pr[0][hq] = p0;
      pr[1][hq] = p1;
      const float l = wave_sum(p0 + p1);
      if (lane == 0) {
        M.rv[wave] = rv;
        M.wstat[wave][hq][0] = m;          // -inf when the wave owns no token
        M.wstat[wave][hq][1] = l;
      }
    }
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) lds_store_f<GQ>(Ssc + (lane + 64 * rep) * GQ, pr[rep]);
    wave_lds_sync();
  }

  // p^T A_V (down-projection of the low-rank Value term) over the wave's rows; wv starts at 0
  {
    float* wv = &M.wv[wave][0][0];
    if (rv == 4) {
      if (rows_lds) lowrank_value_down<GQ, 4, false>(Sav, avr, pr, wv, lane, nw);
      else lowrank_value_down<GQ, 4, true>(Sav, avr, pr, wv, lane, nw);
    } else if (rv == 2) {
      if (rows_lds) lowrank_value_down<GQ, 2, false>(Sav, avr, pr, wv, lane, nw);
      else lowrank_value_down<GQ, 2, true>(Sav, avr, pr, wv, lane, nw);
    } else if (rv == 8) {
      if (rows_lds) lowrank_value_down<GQ, 8, false>(Sav, avr, pr, wv, lane, nw);
      else lowrank_value_down<GQ, 8, true>(Sav, avr, pr, wv, lane, nw);
    } else if (rv > 0) {
      float part[GQ][8];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
        for (int r = 0; r < 8; ++r) part[hq][r] = 0.0f;
#pragma unroll
      for (int rep = 0; rep < 2; ++rep) {
        const int row = lane + 64 * rep;
        if (row < nw) {
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            if (r < rv) {
              const float a = h2f(Sav[row * rv + r]);
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) part[hq][r] += pr[rep][hq] * a;
            }
          }
        }
      }
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          if (r < rv) {
            const float s = wave_sum(part[hq][r]);
            if (lane == 0) wv[hq * 8 + r] = s;
          }
        }
    }
  }

  // =================== Value side on the matrix cores ===================
  floatx4 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
  // operand prep: a lane handles, for its own channel group Gl, pairs of rows of a code block whose fp16
  // halves share a 32-bit word of the operand row (val_slot: rows VD apart inside a block of 2 VD), so every
  // operand store is a whole word; positions and scales are the same for every block
  const int lgNG = (NG == 1) ? 0 : (NG == 2) ? 1 : 2;
  const int Gl = lane & (NG - 1);
  constexpr int VD = (BITS == 2) ? 8 : 4;
  constexpr int NPAIR = TB / 2;                                    // row pairs of a code block
  constexpr int KV = (NPAIR * NG + 63) / 64;                       // pairs per lane (1 or 2)
  int vslot[KV], vrow[KV];
  float vscale[KV];
#pragma unroll
  for (int k = 0; k < KV; ++k) {
    const int pi = (lane >> lgNG) + k * (64 >> lgNG);              // pair index inside the block
    const int t0 = (pi / VD) * (2 * VD) + (pi % VD);               // its rows: t0 and t0 + VD
    int skg, idx, lg;
    val_slot<BITS>(t0 & (TB - 1), skg, idx, lg);
    vrow[k] = pi < NPAIR ? t0 : -1;
    vslot[k] = Gl * 2 * GQ * vop(TB) + skg * (TB / 4) + idx;       // even
    vscale[k] = opscale(lg);
  }
  float pmr[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) pmr[hq] = 0.0f;
#pragma unroll
  for (int bl = 0; bl < VBLK; ++bl) {
    const int tl0 = bl * TB;                       // first row (inside the wave) of this code block
    if (tl0 < nw) {                                // wave-uniform
#pragma unroll
      for (int k = 0; k < KV; ++k) {
        if (vrow[k] >= 0) {
          uint32_t first[GQ];   // (hi, lo) parts of the first row's operand
          _Float16* dst = opnd + vslot[k];
#pragma unroll
          for (int rep = 0; rep < 2; ++rep) {
            const int row = tl0 + vrow[k] + VD * rep;
            const uint32_t sb = row < nw ? Sszv[row * NG + Gl] : 0u;
            const float delta = h2f(sb & 0xFFFFu), mn = h2f(sb >> 16);
            const float ds = delta * vscale[k];
            float ph[GQ];
            lds_load_f<GQ>(Ssc + row * GQ, ph);
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) {
              const float pv = ph[hq];
              const float w = pv * ds;
              const _Float16 hi = (_Float16)w;
              const _Float16 lo = (_Float16)(w - (float)hi);
              pmr[hq] += pv * mn;
              if (rep == 0) {
                first[hq] = pack_f16x2(hi, lo);
              } else {
                const uint32_t second = pack_f16x2(hi, lo);
                *reinterpret_cast<uint32_t*>(dst + (2 * hq) * vop(TB)) = GEAR_BYTE_PERM(second, first[hq], 0x05040100u);
                *reinterpret_cast<uint32_t*>(dst + (2 * hq + 1) * vop(TB)) = GEAR_BYTE_PERM(second, first[hq], 0x07060302u);
              }
            }
          }
        }
      }
      wave_lds_sync();
      for (int G = 0; G < NG; ++G) {
        // (lanes of the unused columns n16 >= 2 GQ read column 0: their output columns are never looked at)
        const _Float16* src = opnd + (size_t)(G * 2 * GQ + (n16 < 2 * GQ ? n16 : 0)) * vop(TB) + kg * (TB / 4);
        const half8 pa0 = __builtin_bit_cast(half8, *reinterpret_cast<const uint4*>(src));
        half8 pa1 = pa0;
        if (BITS == 2) pa1 = __builtin_bit_cast(half8, *reinterpret_cast<const uint4*>(src + 8));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          if ((j >> (lg - 4)) == G) {   // channel tile j (16 channels) lies in group G
            if (BITS == 2) {
              uint32_t v[8];
              Codec<2>::unpack(pin_here(vw[bl][j]), v);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa0, as_half8(v[0], v[1], v[2], v[3]), acc[j], 0, 0, 0);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa1, as_half8(v[4], v[5], v[6], v[7]), acc[j], 0, 0, 0);
            } else {
              uint32_t v[4];
              Codec<4>::unpack(pin_here(vw[bl][j]), v);
              acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(pa0, as_half8(v[0], v[1], v[2], v[3]), acc[j], 0, 0, 0);
            }
          }
            }
      }
      wave_lds_sync();
    }
  }
  // fixed outlier slots of the Value channels lane and lane + 64 in the wave's two tiles (requested here: the
  // reductions and the down-projection below cover their latency, and the registers were needed until now)
  uint2 ellv[2][2];
#pragma unroll
  for (int rep = 0; rep < 2; ++rep)
#pragma unroll
    for (int ti = 0; ti < 2; ++ti) {
      ellv[ti][rep] = make_uint2(0, 0);
      if (dm.ppm > 0 && ti * TILE < nw)
        ellv[ti][rep] = *reinterpret_cast<const uint2*>(
            vs.ell + (((size_t)slab * vs.ntile_cap + tw0 / TILE + ti) * D + lane + 64 * rep) * ELL_V);
    }
  // sum_t p_t zero_V[t][G]: lanes with equal lane % NG hold group G's terms; the four rows
  // of 16 lanes add their sums into pm (zero on entry; groups G >= NG stay 0)
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    float u = pmr[hq];
    if (NG == 1) u += dpp_f<DPP_XOR1>(u);
    if (NG <= 2) u += dpp_f<DPP_XOR2>(u);
    u += dpp_f<DPP_ROR4>(u);
    u += dpp_f<DPP_ROR8>(u);
    if ((lane & 15) < NG) atomicAdd(&M.pm[wave][hq][lane & 15], u);
  }
  // D[col 4*kg + i][channel 16 j + n16] -> this wave's output plane
  {
    const int hq0 = 2 * kg, hq1 = 2 * kg + 1;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float o0 = (acc[j][0] + acc[j][1]) * MFMA_OUT_SCALE, o1 = (acc[j][2] + acc[j][3]) * MFMA_OUT_SCALE;
      if constexpr (GQ == 1) {
        if (kg == 0) Sosp[16 * j + n16] = o0;
      } else {
        if (hq0 < GQ) *reinterpret_cast<float2*>(&Sosp[(16 * j + n16) * GQ + hq0]) = make_float2(o0, o1);
      }
    }
  }

  wave_lds_sync();

  // sparse Value term into this wave's plane.  Fixed slots: the lane owns the channel.
  if (dm.ppm > 0) {
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) {
      const int c = lane + 64 * rep;
      float a2[GQ];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) a2[hq] = 0.0f;
#pragma unroll
      for (int ti = 0; ti < 2; ++ti) {
        const uint32_t es[2] = {ellv[ti][rep].x, ellv[ti][rep].y};
#pragma unroll
        for (int i = 0; i < ELL_V; ++i) {
          const float v = h2f(es[i] >> 16);
          const int row = ti * TILE + (int)(es[i] & 63u);
          float ph[GQ];
          lds_load_f<GQ>(Ssc + row * GQ, ph);
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) a2[hq] += ph[hq] * v;
        }
      }
      float oh[GQ];
      lds_load_f<GQ>(Sosp + c * GQ, oh);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) oh[hq] += a2[hq];
      lds_store_f<GQ>(Sosp + c * GQ, oh);
    }
    wave_lds_sync();
    auto add_v = [&](uint32_t en) {
      const int row = (en & 0xFFFFu) >> 7, c = en & 127u;
      const float v = h2f(en >> 16);
      float ph[GQ];
      lds_load_f<GQ>(Ssc + row * GQ, ph);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) atomicAdd(&Sosp[c * GQ + hq], ph[hq] * v);
    };
#pragma unroll
    for (int i = 0; i < SPR; ++i)
      if ((uint32_t)(lane + 64 * i) < cv0 + cv1) add_v(spv_r[i]);
    for (uint32_t e = SPR * 64 + lane; e < cv0 + cv1; e += 64) {
      const bool second = e >= cv0;
      const uint32_t en = second ? poolv[ov1 + (e - cv0)] : poolv[ov0 + e];
      add_v(en + (second ? TILE * D : 0));
    }
    wave_lds_sync();
  }
  block_lds_sync();

  // =================== merge the four waves' states, write the record ===================
  // (an empty wave has m = -inf and weight 0; its plane, pm and wv hold zeros)
  const bool one_b = shared_b && (rv == 0 || rv == 2 || rv == 4 || rv == 8);   // block-uniform: one B_V, one read per row
  for (int i = tid; i < GQ * D; i += 256) {
    const int c = i / GQ, hq = i % GQ, G = c >> lg;   // the lanes of a wave read consecutive plane entries
    float mw[4], lw[4], f[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float2 st = *reinterpret_cast<const float2*>(&M.wstat[w][hq][0]);
      mw[w] = st.x;
      lw[w] = st.y;
    }
    const float Mx = fmaxf(fmaxf(mw[0], mw[1]), fmaxf(mw[2], mw[3]));
#pragma unroll
    for (int w = 0; w < 4; ++w) f[w] = mw[w] == -INFINITY ? 0.0f : __expf(mw[w] - Mx);
    float o = 0.0f, l = 0.0f;
    if (one_b) {
      // sum_w f_w (plane_w + pm_w) + B_V[c] . (sum_w f_w wv_w): every load is independent of the others
      float t[8];
#pragma unroll
      for (int r = 0; r < 8; ++r) t[r] = 0.0f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float* plane = reinterpret_cast<const float*>(smem + L.wave0 + (size_t)w * L.wave_stride + L.osp);
        o += f[w] * (plane[c * GQ + hq] + M.pm[w][hq][G]);
        l += f[w] * lw[w];
        if (rv > 0) {
          const float4 a = *reinterpret_cast<const float4*>(&M.wv[w][hq][0]);
          t[0] += f[w] * a.x; t[1] += f[w] * a.y; t[2] += f[w] * a.z; t[3] += f[w] * a.w;
        }
        if (rv > 4) {
          const float4 a = *reinterpret_cast<const float4*>(&M.wv[w][hq][4]);
          t[4] += f[w] * a.x; t[5] += f[w] * a.y; t[6] += f[w] * a.z; t[7] += f[w] * a.w;
        }
      }
      if (rv == 4) {
        float bb[4];
        lds_row_f16<4>(Sbfv + c * 4, bb);
#pragma unroll
        for (int r = 0; r < 4; ++r) o += t[r] * bb[r];
      } else if (rv == 2) {
        float bb[2];
        lds_row_f16<2>(Sbfv + c * 2, bb);
        o += t[0] * bb[0] + t[1] * bb[1];
      } else if (rv == 8) {
        float bb[8];
        lds_row_f16<8>(Sbfv + c * 8, bb);
#pragma unroll
        for (int r = 0; r < 8; ++r) o += t[r] * bb[r];
      }
    } else {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        if (mw[w] == -INFINITY) continue;
        const float* plane = reinterpret_cast<const float*>(smem + L.wave0 + (size_t)w * L.wave_stride + L.osp);
        float ow = plane[c * GQ + hq] + M.pm[w][hq][G];
        const uint16_t* bfw = reinterpret_cast<const uint16_t*>(smem + L.bf + (shared_b ? L.bf_v0 : w * L.bf_cw + L.bf_vc));
        const int rvw = GEAR_WAVE_UNIFORM(M.rv[w]);
        const float* wvw = &M.wv[w][hq][0];
        if (rvw == 4) {
          float bb[4];
          lds_row_f16<4>(bfw + c * 4, bb);
#pragma unroll
          for (int r = 0; r < 4; ++r) ow += wvw[r] * bb[r];
        } else if (rvw == 2) {
          float bb[2];
          lds_row_f16<2>(bfw + c * 2, bb);
          ow += wvw[0] * bb[0] + wvw[1] * bb[1];
        } else if (rvw == 8) {
          float bb[8];
          lds_row_f16<8>(bfw + c * 8, bb);
#pragma unroll
          for (int r = 0; r < 8; ++r) ow += wvw[r] * bb[r];
        } else {
          for (int r = 0; r < rvw; ++r) ow += wvw[r] * h2f(bfw[c * rvw + r]);
        }
        o += f[w] * ow;
        l += f[w] * lw[w];
      }
    }
    float* rec = rec_base + (size_t)hq * rec_stride;
    rec[2 + c] = o;
    if (c == 0) {
      rec[0] = Mx;
      rec[1] = l;
    }
  }
}

}  // namespace gear
