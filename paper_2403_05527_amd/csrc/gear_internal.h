// Internal definitions shared by the HIP translation units of libgear:
// the private arena layout, kernel argument structs and small device helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>

#include "gear.h"

// Declares the kernel's dynamically sized LDS array (a build that runs the
// kernels elsewhere than on the GPU may predefine this).
#ifndef GEAR_DYN_LDS
#define GEAR_DYN_LDS(name) extern __shared__ __align__(16) unsigned char name[]
#endif

// Tells the compiler that an integer is the same in every lane of the wave (it is
// then kept in a scalar register and branches on it are scalar branches).
#ifndef GEAR_WAVE_UNIFORM
#define GEAR_WAVE_UNIFORM(x) __builtin_amdgcn_readfirstlane(x)
#endif

// An empty volatile asm that takes and returns a value in a vector register: the
// compiler can neither hoist nor sink what depends on it.
#ifndef GEAR_PIN_VGPR
#define GEAR_PIN_VGPR(x) asm volatile("" : "+v"(x))
#endif

// Block barrier that orders LDS traffic only.  __syncthreads() also drains every
// outstanding global load and store of the wave (loads and stores share one
// counter on this chip), which would serialise prefetched loads with the barrier;
// none of the kernels exchanges data between threads of a block through global
// memory, so LDS ordering is all they need.
#ifndef GEAR_LDS_BARRIER
#define GEAR_LDS_BARRIER()                                              \
  do {                                                                  \
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");     \
    __builtin_amdgcn_s_barrier();                                       \
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");     \
  } while (0)
#endif

// v_perm_b32: byte i of the result is byte sel.byte[i] of the 8 bytes {hi, lo}
// (0..3 = bytes of lo, 4..7 = bytes of hi, 0x0c = zero).
#ifndef GEAR_BYTE_PERM
#define GEAR_BYTE_PERM(hi, lo, sel) __builtin_amdgcn_perm((hi), (lo), (sel))
#endif
// v_bfe_u32: `width` bits of x from bit `off`
#ifndef GEAR_UBFE
#define GEAR_UBFE(x, off, width) __builtin_amdgcn_ubfe((x), (off), (width))
#endif
// v_med3_f32: the median of three = x clamped to [lo, hi]
#ifndef GEAR_FMED3
#define GEAR_FMED3(x, lo, hi) __builtin_amdgcn_fmed3f((x), (lo), (hi))
#endif

// Raw buffer views: a load whose bytes do not all lie below the view's size returns 0,
// so a ragged tail needs neither a per-lane test nor a 64-bit address per lane.
// Fewest tokens (B * n) of a call for which the Value selection runs by token rows, four tokens per wave
// (below that a flushed buffer's few tokens take one wave each).  The CPU stand-in lowers it so that its small
// cases reach those kernels.
#ifndef GEAR_ROWS_MIN_TOKENS
#define GEAR_ROWS_MIN_TOKENS 16384
#endif
#ifndef GEAR_BUF_T
#define GEAR_BUF_T __amdgpu_buffer_rsrc_t
#define GEAR_BUF_MAKE(p, bytes) \
  __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(static_cast<const void*>(p)), 0, (int)(bytes), 0x00020000)
#define GEAR_BUF_LOAD8(b, off) __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64((b), (int)(off), 0, 0))
#define GEAR_BUF_LOAD16(b, off) __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128((b), (int)(off), 0, 0))
// the same with the non-temporal hint (data that is read once)
#define GEAR_BUF_LOAD16_NT(b, off) __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128((b), (int)(off), 0, 2))
#define GEAR_BUF_LOAD4(b, off) ((uint32_t)__builtin_amdgcn_raw_buffer_load_b32((b), (int)(off), 0, 0))
#define GEAR_BUF_LOAD2(b, off) ((uint32_t)__builtin_amdgcn_raw_buffer_load_b16((b), (int)(off), 0, 0))
// a store that does not lie wholly inside the view is dropped; non-temporal (data written once, read by a later kernel)
#define GEAR_BUF_STORE16_NT(b, off, v) \
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(gear::u32x4_t, (v)), (b), (int)(off), 0, 2)
#define GEAR_BUF_STORE4(b, off, v) __builtin_amdgcn_raw_buffer_store_b32((uint32_t)(v), (b), (int)(off), 0, 0)
#define GEAR_BUF_STORE2(b, off, v) __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(v), (b), (int)(off), 0, 0)
#endif

namespace gear {

typedef float floatx4 __attribute__((ext_vector_type(4)));   // MFMA accumulator tile of one lane

constexpr int D = 128;      // head dimension
constexpr int TILE = 64;    // tokens per sparse-list tile
constexpr int VPOOL_FIXED = 48;   // entries of the reserved list region of one Value (head, tile)
constexpr int ELL_K = 4;    // fixed outlier slots per Key token row
constexpr int ELL_V = 2;    // fixed outlier slots per Value channel and tile
constexpr uint32_t ELL_VALID = 0x8000u;

// ---------------------------------------------------------------------------
// Filter_s thresholds of one vector (Eq. 4).  An entry with monotone key `k`
// and in-vector index `i` is an outlier iff
//   k > tau_top || (k == tau_top && i <= i_top) ||
//   k < tau_bot || (k == tau_bot && l_bot < i && i <= i_bot).
// ---------------------------------------------------------------------------
struct Thresh {
  uint32_t tau_top;
  int32_t i_top;
  uint32_t tau_bot;
  int32_t i_bot;
  int32_t l_bot;
  int32_t pad[3];
};

// Geometry shared by all kernels of one cache.
struct Dims {
  int B, H, Hq;
  int bits;   // b
  int g;      // group size (128 with the per-vector grouping: what the tiles of the Value kernels and of the decode use)
  int kcvt;   // per-vector grouping: one Key group per segment, one Value group per token over all heads
  int vhead;  // Filter_s of the Values per head
  int ppm;    // outlier ratio in parts per million
  int wpr;    // 32-bit words per Key code row (128*b/32)
  int tpw;    // tokens per Value code word (32/b)
  float qmax; // 2^b - 1
};

// One tensor (K or V) of one stored segment.  Private physical layout:
//  Keys   codes : [slab][n_cap][wpr] u32, token-major rows, channel c at bits
//                 (c % (32/b))*b of word c*b/32.
//  Values codes : [slab][nblk_cap][512] u32 in blocks of 4*tpw tokens; word
//                 (kg*16 + c%16)*8 + c/16 of a block holds channel c for the tpw
//                 tokens 4*tpw*blk + tpw*kg + i at bits i*b (the order in which
//                 the decode kernel's MFMA B operand consumes them).
//  sz           : (scale, zero) as two fp16 in one u32 (scale low half).
//                 Keys [slab][ng_cap][128]; Values [slab][n_cap][128/g].
//  A, Bf        : fp16 [slab][n_cap][rank], [slab][128][rank].
//  ell          : the sparse matrix S (Filter_s, Eq. 4), fixed-slot part.  Keys:
//                 [slab][n_cap][4] u32, the first 4 outliers of a token row in
//                 channel order, slot = c | 0x8000 | fp16 value << 16.  Values:
//                 [slab][ntile_cap][128][2] u32, the first 2 outliers of one
//                 channel inside a 64-token tile in token order, slot =
//                 (t % 64) | 0x8000 | value << 16.  An empty slot is 0.  A reader
//                 that owns the row (Keys) / the channel (Values) sums its slots
//                 without any exchange with other lanes.
//  sp_table     : [slab][ntile_cap] (offset, count) of the tile's overflow list:
//                 the outliers that found no slot.
//  sp_pool      : u32 entries (low 16 bits: (t % 64)*128 + c, high 16: fp16
//                 value).  Keys: one pool per slab, lists ordered (t, c);
//                 Values: one pool per batch element, lists ordered (c, t).  A Value
//                 pool starts with one reserved region of VPOOL_FIXED entries per
//                 (head, tile), at (head * ntile_cap + tile) * VPOOL_FIXED: a list that
//                 fits lies there and needs no allocation; longer lists are
//                 allocated behind the reserved regions from a counter per batch
//                 element (every tile of 32 heads bumping one counter costs more
//                 than the rest of the kernel's list handling).
struct SegView {
  uint32_t* codes;
  uint32_t* sz;
  uint16_t* A;
  uint16_t* Bf;
  uint32_t* ell;
  uint2* sp_table;
  uint32_t* sp_pool;
  int n;         // tokens stored
  int n_cap;     // token capacity of this region
  int rank;
  int ng_cap;    // Key groups capacity
  int nblk_cap;  // Value code blocks capacity
  int ntile_cap;
  uint32_t pool_cap;  // entries per slab (Keys) / per batch element (Values)
  int t0;        // first token of this segment in the whole cache
  int g0;        // first Key group of this segment in the whole cache
};
// Key group of token t of a segment
__host__ __device__ inline int key_group(const Dims& dm, int t) { return dm.kcvt ? 0 : t / dm.g; }

// ---------------------------------------------------------------------------
// fp16 helpers (bit patterns travel as integers)
// ---------------------------------------------------------------------------
__device__ __forceinline__ float h2f(uint32_t bits16) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}
__device__ __forceinline__ uint32_t f2h(float f) {  // round to nearest even
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
// Monotone 16-bit key of an fp16 bit pattern; -0 and +0 share one key.
__device__ __forceinline__ uint32_t key16(uint32_t h) {
  h &= 0xFFFFu;
  return (h & 0x8000u) ? ((0u - h) & 0xFFFFu) : (h | 0x8000u);
}
// The same key for two fp16 values packed in one 32-bit word (negative: two's
// complement of the pattern, which also maps -0 onto +0's key; positive: + 0x8000).
__device__ __forceinline__ uint32_t key16x2(uint32_t h2) {
  typedef short i16x2_t __attribute__((ext_vector_type(2)));
  typedef unsigned short k16x2_t __attribute__((ext_vector_type(2)));
  const uint32_t s = __builtin_bit_cast(uint32_t, __builtin_bit_cast(i16x2_t, h2) >> 15);   // 0xFFFF over a negative half
  const uint32_t x = h2 ^ (s | 0x80008000u);                                                // negative: ~h, positive: h + 0x8000
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(k16x2_t, x) - __builtin_bit_cast(k16x2_t, s));   // negative: ~h + 1
}
// Loads and stores of data that is touched once per kernel and is larger than the
// caches (non-temporal: the lines are not kept).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream16(void* p, uint4 v) {
  u32x4_t x = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(x, reinterpret_cast<u32x4_t*>(p));
}
// fp16 bit pattern of a key (the key of +-0 gives +0)
__device__ __forceinline__ uint32_t unkey16(uint32_t k) {
  return (k & 0x8000u) ? (k & 0x7FFFu) : ((0u - k) & 0xFFFFu);
}
// two unsigned 16-bit lanes per 32-bit word
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2_t, a), __builtin_bit_cast(u16x2_t, b)));
}
__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, a), __builtin_bit_cast(u16x2_t, b)));
}
// fp16 entry e (0..7) of a row piece of four words
// (the words are passed by value: selecting between elements of an array in place is
// compiled into an indexed load, which moves the array to scratch memory)
__device__ __forceinline__ uint32_t half_of(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, int e) {
  const uint32_t w01 = (e & 2) ? w1 : w0, w23 = (e & 2) ? w3 : w2;
  const uint32_t w = (e & 4) ? w23 : w01;
  return (w >> ((e & 1) * 16)) & 0xFFFFu;
}
// The predicate of Thresh as two 32-bit compares.  With cT = key << 16 | (0xFFFF - idx)
// (larger key first, then smaller index) and cB = key << 16 | idx, an entry is an
// outlier iff cT >= top || cB < bot.  The l_bot bound needs no term of its own: it
// is set only where top and bottom share one threshold value, and there the entries
// it excludes (idx <= l_bot = i_top) are top outliers anyway.  Needs idx <= 0xFFFF
// and finite inputs (keys <= 0xFC00), which the entry points guarantee.
struct ThreshPair {
  uint32_t top, bot;
};
__device__ __forceinline__ ThreshPair pack_thresh(const Thresh& th) {
  ThreshPair p;
  if (th.tau_top > 0xFFFFu) {
    p.top = 0xFFFFFFFFu;                                   // no top outliers
  } else {
    const uint32_t lo = th.i_top < 0 ? 0x10000u : (th.i_top > 0xFFFF ? 0u : 0xFFFFu - (uint32_t)th.i_top);
    p.top = (th.tau_top << 16) + lo;
  }
  const uint32_t lob = th.i_bot < 0 ? 0u : (th.i_bot >= 0xFFFF ? 0x10000u : (uint32_t)th.i_bot + 1u);
  p.bot = (th.tau_bot << 16) + lob;
  return p;
}
__device__ __forceinline__ Thresh thresh_none() {
  Thresh th;
  th.tau_top = 0x10000u;
  th.i_top = -1;
  th.tau_bot = 0u;
  th.i_bot = -1;
  th.l_bot = -1;
  th.pad[0] = th.pad[1] = th.pad[2] = 0;
  return th;
}

// ---------------------------------------------------------------------------
// Group quantizer (Eq. 2).  The integer code is decided in fp32 with this exact
// operation sequence: delta32 = (mx - mn) / qmax; delta = fp16(delta32);
// inv = 1 / delta; t = (y - mn) * inv; code = clamp(rint(t), 0, qmax).
// ---------------------------------------------------------------------------
struct GroupQ {
  float mn;     // zero-point (an fp16 value)
  float delta;  // fp16-rounded scale, as float
  float inv;    // 1/delta, 0 when delta == 0
};
// (The decision sequence is kept free of fused multiply-adds whatever the compiler's default is:
// contraction is switched off inside these functions and around the quantizer loops of the kernels.)
__device__ __forceinline__ GroupQ make_group(float mn, float mx, float qmax) {
#pragma clang fp contract(off)
  GroupQ q;
  q.mn = mn + 0.0f;  // -0 -> +0
  mx = mx + 0.0f;
  float d32 = __fdiv_rn(__fsub_rn(mx, q.mn), qmax);
  q.delta = h2f(f2h(d32));
  q.inv = q.delta > 0.0f ? __fdiv_rn(1.0f, q.delta) : 0.0f;
  return q;
}
// 1 / d, correctly rounded, for a d > 0 that is an fp16 value (11 significant bits): the hardware's
// reciprocal estimate (within 1 ulp) refined by one Newton step.  The residual 1 - d r of the estimate
// is exact in fp32 (12 significant bits after the cancellation) and the step leaves a relative error
// of about 2^-46, far below the distance (at least 2^-36, relative) of a quotient 2^k / m, m < 2^11,
// from the nearest rounding boundary: the same float as the IEEE division, in 3 instructions.
__device__ __forceinline__ float recip_of_half(float d) {
  const float r = __builtin_amdgcn_rcpf(d);
  return __builtin_fmaf(__builtin_fmaf(-d, r, 1.0f), r, r);
}
__device__ __forceinline__ GroupQ load_group(uint32_t sz_bits) {
  GroupQ q;
  q.delta = h2f(sz_bits & 0xFFFFu);
  q.mn = h2f(sz_bits >> 16);
  q.inv = q.delta > 0.0f ? recip_of_half(q.delta) : 0.0f;   // = 1 / delta as the quantizer computed it
  return q;
}
__device__ __forceinline__ uint32_t group_bits(const GroupQ& q) {
  return f2h(q.delta) | (f2h(q.mn) << 16);
}
// Byte 0 of four words in one word (codes and the like read off float mantissas).
__device__ __forceinline__ uint32_t low_bytes4(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3) {
  return GEAR_BYTE_PERM(GEAR_BYTE_PERM(b3, b2, 0x0c0c0400u), GEAR_BYTE_PERM(b1, b0, 0x0c0c0400u), 0x05040100u);
}
__device__ __forceinline__ float clamp_f32(float x, float lo, float hi) { return GEAR_FMED3(x, lo, hi); }
// Quantization error of one entry (Alg. 1: R = Y - D-hat, D-hat = code * scale + zero) with
// the code decided by the quantizer's own operation sequence (Eq. 2), so it is the stored one.
__device__ __forceinline__ float quant_error(float y, float mn, float inv, float delta, float qmax) {
#pragma clang fp contract(off)
  const float ym = __fsub_rn(y, mn);
  const float c = clamp_f32(rintf(__fmul_rn(ym, inv)), 0.0f, qmax);
  return __builtin_fmaf(-c, delta, ym);
}

// Start matrix B0 of Algorithm 2 (its "random_initialize"), as the caller's array or drawn here.
// Entry i of the [2 (K, V), B, H, 128, rank] array is u(seed, i) = ((z >> 40) - 2^23) / 2^23 with
// z = the 64-bit mix below of seed + (i + 1) * 0x9E3779B97F4A7C15 (the SplitMix64 step): integers
// only, uniform on a 24-bit grid in [-1, 1), so any implementation of the same formula gives the
// same floats.
struct StartB {
  const float* init;   // device fp32 [slabs of this tensor][128][rank], or nullptr: draw
  uint64_t seed;
  uint64_t base;       // index of this tensor's first entry in the whole array
};
__host__ __device__ inline float start_entry(uint64_t seed, uint64_t i) {
  uint64_t z = seed + 0x9E3779B97F4A7C15ull * (i + 1ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z ^= z >> 31;
  return (float)((int)(z >> 40) - (1 << 23)) * (1.0f / 8388608.0f);
}
__device__ __forceinline__ float start_b(const StartB& sb, int slab, int c, int rank, int r) {
  const uint64_t i = ((uint64_t)slab * D + c) * rank + r;
  return sb.init ? sb.init[i] : start_entry(sb.seed, sb.base + i);
}

__device__ __forceinline__ void block_lds_sync() { GEAR_LDS_BARRIER(); }

// ---------------------------------------------------------------------------
// wavefront (64 lanes) primitives
// ---------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Data-parallel-primitive (DPP) lane exchanges: one VALU op each, no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141; // lane i <-> 7 - i inside each group of 8
constexpr int DPP_MIRROR = 0x140;      // lane i <-> 15 - i inside each row of 16

// Sum / max over each row of 16 lanes, result in every lane of the row.
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f<DPP_XOR1>(v);
  v += dpp_f<DPP_XOR2>(v);
  v += dpp_f<DPP_HALF_MIRROR>(v);
  v += dpp_f<DPP_MIRROR>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_f<DPP_XOR1>(v));
  v = fmaxf(v, dpp_f<DPP_XOR2>(v));
  v = fmaxf(v, dpp_f<DPP_HALF_MIRROR>(v));
  v = fmaxf(v, dpp_f<DPP_MIRROR>(v));
  return v;
}
// Sums of several per-lane values over a row of 16 lanes in one go: the first exchanges
// halve the number of values a lane carries instead of summing each value separately.
// Lane l returns the row's sum of v[l & 3] (sum4) or v[l & 1] (sum2).
constexpr int DPP_ROR4 = 0x124, DPP_ROR8 = 0x128;   // rotate by 4 / 8 lanes inside a row of 16
__device__ __forceinline__ float row16_sum4(float v0, float v1, float v2, float v3, int lane) {
  const bool b0 = (lane & 1) != 0, b1 = (lane & 2) != 0;
  const float t0 = (b0 ? v1 : v0) + dpp_f<DPP_XOR1>(b0 ? v0 : v1);
  const float t1 = (b0 ? v3 : v2) + dpp_f<DPP_XOR1>(b0 ? v2 : v3);
  float u = (b1 ? t1 : t0) + dpp_f<DPP_XOR2>(b1 ? t0 : t1);
  u += dpp_f<DPP_ROR4>(u);
  u += dpp_f<DPP_ROR8>(u);
  return u;
}
__device__ __forceinline__ float row16_sum2(float v0, float v1, int lane) {
  const bool b0 = (lane & 1) != 0;
  float u = (b0 ? v1 : v0) + dpp_f<DPP_XOR1>(b0 ? v0 : v1);
  u += dpp_f<DPP_XOR2>(u);
  u += dpp_f<DPP_ROR4>(u);
  u += dpp_f<DPP_ROR8>(u);
  return u;
}

__device__ __forceinline__ float lane_bcast(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}
// Sum / max over the 64 lanes, result in every lane (wave-uniform).  After the sums inside the rows of
// 16, lane 15 of rows 0 and 2 is added into rows 1 and 3 (row_bcast:15), then lane 31 into rows 2 and 3
// (row_bcast:31): lane 63 holds (r2 + r3) + (r0 + r1), which one scalar read spreads to the wave.
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_rows_f(float old, float v) {   // rows outside ROW_MASK (and lanes without a source) keep `old`
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  v += dpp_rows_f<DPP_ROW_BCAST15, 0xA>(0.0f, v);
  v += dpp_rows_f<DPP_ROW_BCAST31, 0xC>(0.0f, v);
  return lane_bcast(v, 63);
}
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  v = fmaxf(v, dpp_rows_f<DPP_ROW_BCAST15, 0xA>(-INFINITY, v));
  v = fmaxf(v, dpp_rows_f<DPP_ROW_BCAST31, 0xC>(-INFINITY, v));
  return lane_bcast(v, 63);
}
template <typename T>
__device__ __forceinline__ T wave_sum_shfl(T v) {  // generic (integers, doubles)
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Orders this wave's earlier LDS writes before LDS reads by other lanes of the
// same wave (the LDS executes one wave's operations in order, so only the
// compiler has to be stopped from moving them).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// inclusive prefix sum over lanes
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  const int lane = lane_id();
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_up(v, o, 64);
    if (lane >= o) v += t;
  }
  return v;
}
__device__ __forceinline__ uint32_t wave_incl_suffix(uint32_t v) {
  const int lane = lane_id();
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    uint32_t t = __shfl_down(v, o, 64);
    if (lane + o < 64) v += t;
  }
  return v;
}

}  // namespace gear
