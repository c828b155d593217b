// Filter_s thresholds (Eq. 4) of FOUR vectors per wavefront, one per row of 16 lanes: the selection of
// gear_select.h at row granularity, for vectors of at most 1024 entries (Value token rows of models with
// up to eight KV heads).  For such short vectors the cost of a selection is mostly per vector (histogram
// clears, scans, tie search), not per entry; four selections that run side by side in one wave share it.
//
// Lane i of a row holds the vector as eight chunks of 8 keys: chunk h, entry e <-> in-vector index
// 128 h + 8 i + e (head h, channel 8 i + e of a Value token row).  Same algorithm, same results as
// wave_select: two-level radix select on the 16-bit monotone keys (high byte, low byte) with the row's own
// LDS histograms, then the index cut among the entries equal to a threshold (the lower index wins; when
// top and bottom share one threshold value the bottom set continues where the top set stopped).
#pragma once
#include <climits>
#include "gear_internal.h"
#include "gear_select.h"

namespace gear {

constexpr int SELECT_ROW_LDS_WORDS = 512;   // LDS words per vector (row of 16 lanes)

// Lane exchanges inside a row of 16 with zero fill: lane i reads lane i + N (row_shl) or i - N (row_shr);
// a lane without a source reads 0.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u_zero(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ uint32_t row16_incl_suffix(uint32_t v) {   // sum over lanes i .. 15 of the row
  v += dpp_u_zero<0x101>(v);
  v += dpp_u_zero<0x102>(v);
  v += dpp_u_zero<0x104>(v);
  v += dpp_u_zero<0x108>(v);
  return v;
}
__device__ __forceinline__ uint32_t row16_incl_prefix(uint32_t v) {   // sum over lanes 0 .. i of the row
  v += dpp_u_zero<0x111>(v);
  v += dpp_u_zero<0x112>(v);
  v += dpp_u_zero<0x114>(v);
  v += dpp_u_zero<0x118>(v);
  return v;
}
// bit j: the predicate of lane j of my row
__device__ __forceinline__ uint32_t row16_ballot(bool p) {
  const unsigned long long m = __ballot(p);
  return (uint32_t)(m >> (lane_id() & 48)) & 0xFFFFu;
}
__device__ __forceinline__ uint32_t row16_get(uint32_t v, int src) { return (uint32_t)__shfl((int)v, src, 16); }

// h: the row's 256 counters in LDS.  The bin where the count taken from the top reaches k (k >= 1), and
// `above` = entries in bins strictly above it.  Lane i looks at bins 16 i .. 16 i + 15.
__device__ __forceinline__ void row_scan_from_top(const uint32_t* h, uint32_t k, int& bin, uint32_t& above) {
  const int i = lane_id() & 15;
  uint32_t hh[16];
#pragma unroll
  for (int j = 0; j < 16; j += 4) {
    const uint4 t = *reinterpret_cast<const uint4*>(h + 16 * i + j);
    hh[j] = t.x; hh[j + 1] = t.y; hh[j + 2] = t.z; hh[j + 3] = t.w;
  }
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += hh[j];
  const uint32_t suf = row16_incl_suffix(s);
  const uint32_t m = row16_ballot(suf >= k);   // lanes 0 .. L of the row
  const int L = m ? 31 - __clz((int)m) : 0;
  uint32_t cum = suf - s, ab = cum;
  int bsel = 16 * i;
  bool done = false;
#pragma unroll
  for (int j = 15; j >= 0; --j) {
    const bool hit = !done && cum + hh[j] >= k;
    bsel = hit ? 16 * i + j : bsel;
    ab = hit ? cum : ab;
    done = done || hit;
    cum += done ? 0u : hh[j];
  }
  bin = (int)row16_get((uint32_t)bsel, L);
  above = row16_get(ab, L);
}
__device__ __forceinline__ void row_scan_from_bottom(const uint32_t* h, uint32_t k, int& bin, uint32_t& below) {
  const int i = lane_id() & 15;
  uint32_t hh[16];
#pragma unroll
  for (int j = 0; j < 16; j += 4) {
    const uint4 t = *reinterpret_cast<const uint4*>(h + 16 * i + j);
    hh[j] = t.x; hh[j + 1] = t.y; hh[j + 2] = t.z; hh[j + 3] = t.w;
  }
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) s += hh[j];
  const uint32_t pre = row16_incl_prefix(s);
  const uint32_t m = row16_ballot(pre >= k);   // lanes L .. 15 of the row
  const int L = m ? __ffs((int)m) - 1 : 15;
  uint32_t cum = pre - s, be = cum;
  int bsel = 16 * i + 15;
  bool done = false;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const bool hit = !done && cum + hh[j] >= k;
    bsel = hit ? 16 * i + j : bsel;
    be = hit ? cum : be;
    done = done || hit;
    cum += done ? 0u : hh[j];
  }
  bin = (int)row16_get((uint32_t)bsel, L);
  below = row16_get(be, L);
}

// Index of the m-th entry (in index order, m >= 1) of the row's vector that equals tau; rows with m == 0
// take no part (their result is INT_MAX).  x: the lane's eight chunks; H: chunks in use (N = 128 H).
__device__ __forceinline__ int row_kth_equal(const uint4 (&x)[8], int H, uint32_t tau, uint32_t m) {
  const int i = lane_id() & 15;
  int found = INT_MAX;
  uint32_t base_cnt = 0;
  bool have = m == 0u;
#pragma unroll
  for (int h = 0; h < 8; ++h) {
    if (h < H) {   // wave-uniform
      uint32_t c = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) c += slot16(x[h], e) == tau ? 1u : 0u;
      const uint32_t inc = row16_incl_prefix(c);
      const uint32_t total = row16_get(inc, 15);
      const bool here = !have && base_cnt + total >= m;   // the same in the 16 lanes of a row
      const uint32_t exc = base_cnt + inc - c;
      const bool mine = here && exc < m && m <= base_cnt + inc;
      int idx = INT_MAX;
      uint32_t r = exc;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const bool eq = slot16(x[h], e) == tau;
        r += eq ? 1u : 0u;
        idx = (eq && r == m && idx == INT_MAX) ? 128 * h + 8 * i + e : idx;
      }
      const uint32_t bm = row16_ballot(mine);
      const int got = (int)row16_get((uint32_t)idx, bm ? __ffs((int)bm) - 1 : 0);
      found = here ? got : found;
      have = have || here;
      base_cnt += total;
    }
  }
  return found;
}

// hist: SELECT_ROW_LDS_WORDS u32 of LDS private to the calling row.  All 64 lanes of the wave call together
// (the four rows run in lock step; a row whose token does not exist passes zeros and ignores the result).
// H: heads (chunks) in use, 1..8; the vector has N = 128 H entries.
__device__ __forceinline__ Thresh row_select(const uint4 (&x)[8], int H, int k_top, int k_bot, uint32_t* hist) {
  const int lane = lane_id(), i = lane & 15;
  Thresh th = thresh_none();

  // ---- level 1: histogram of the high key byte
#pragma unroll
  for (int j = 0; j < 256; j += 64) *reinterpret_cast<uint4*>(hist + j + 4 * i) = make_uint4(0, 0, 0, 0);
  wave_lds_sync();
#pragma unroll
  for (int h = 0; h < 8; ++h)
    if (h < H) {
#pragma unroll
      for (int e = 0; e < 8; ++e) atomicAdd(&hist[slot16(x[h], e) >> 8], 1u);
    }
  wave_lds_sync();
  int bin_t = -1, bin_b = -1;
  uint32_t need_t = 0, need_b = 0;
  if (k_top > 0) {
    uint32_t above;
    row_scan_from_top(hist, (uint32_t)k_top, bin_t, above);
    need_t = (uint32_t)k_top - above;
  }
  if (k_bot > 0) {
    uint32_t below;
    row_scan_from_bottom(hist, (uint32_t)k_bot, bin_b, below);
    need_b = (uint32_t)k_bot - below;
  }
  wave_lds_sync();

  // ---- level 2: histograms of the low key byte inside the two boundary bins (only the lanes with an entry
  // in one of them take part in an add)
#pragma unroll
  for (int j = 0; j < 512; j += 64) *reinterpret_cast<uint4*>(hist + j + 4 * i) = make_uint4(0, 0, 0, 0);
  wave_lds_sync();
#pragma unroll
  for (int h = 0; h < 8; ++h)
    if (h < H) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t k = slot16(x[h], e);
        const int hi = (int)(k >> 8);
        const bool in_t = hi == bin_t, in_b = hi == bin_b;
        if (in_t || in_b) atomicAdd(&hist[(in_t ? 0u : 256u) + (k & 255u)], 1u);
      }
    }
  wave_lds_sync();
  if (bin_t == bin_b && bin_t >= 0) {   // one bin holds both thresholds: its entries count for both
#pragma unroll
    for (int j = 0; j < 256; j += 64)
      *reinterpret_cast<uint4*>(hist + 256 + j + 4 * i) = *reinterpret_cast<const uint4*>(hist + j + 4 * i);
  }
  wave_lds_sync();
  uint32_t need_eq_t = 0, cnt_eq_t = 0, need_eq_b = 0, cnt_eq_b = 0;
  if (k_top > 0) {
    int lo;
    uint32_t above;
    row_scan_from_top(hist, need_t, lo, above);
    th.tau_top = ((uint32_t)bin_t << 8) | (uint32_t)lo;
    need_eq_t = need_t - above;
    cnt_eq_t = hist[lo];
  }
  if (k_bot > 0) {
    int lo;
    uint32_t below;
    row_scan_from_bottom(hist + 256, need_b, lo, below);
    th.tau_bot = ((uint32_t)bin_b << 8) | (uint32_t)lo;
    need_eq_b = need_b - below;
    cnt_eq_b = hist[256 + lo];
  }
  wave_lds_sync();

  // ---- ties: among entries equal to the threshold the lowest indices win; when top and bottom share
  // one threshold value the bottom set continues where the top set stopped
  const bool shared = k_top > 0 && k_bot > 0 && th.tau_top == th.tau_bot;
  uint32_t m1, m2, tau2;
  if (shared) {
    m1 = need_eq_t;
    m2 = (need_eq_t + need_eq_b == cnt_eq_t) ? 0u : need_eq_t + need_eq_b;
    tau2 = th.tau_top;
  } else {
    m1 = (k_top > 0 && need_eq_t != cnt_eq_t) ? need_eq_t : 0u;
    m2 = (k_bot > 0 && need_eq_b != cnt_eq_b) ? need_eq_b : 0u;
    tau2 = th.tau_bot;
  }
  int i1 = INT_MAX, i2 = INT_MAX;
  if (__ballot(m1 != 0u) != 0ull) i1 = row_kth_equal(x, H, th.tau_top, m1);   // (wave-uniform: rarely needed)
  if (__ballot(m2 != 0u) != 0ull) i2 = row_kth_equal(x, H, tau2, m2);
  if (k_top > 0) th.i_top = i1;
  if (k_bot > 0) th.i_bot = i2;
  if (shared) th.l_bot = th.i_top;
  return th;
}

}  // namespace gear
