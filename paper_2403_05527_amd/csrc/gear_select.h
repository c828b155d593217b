// Exact top-k / bottom-k selection of one fp16 vector by one wavefront
// (Filter_s of Eq. 4): two-level radix select on the 16-bit monotone key
// (high byte, then low byte), then a tie cutoff by index among the entries that
// equal the threshold.  The result is the Thresh predicate of gear_internal.h,
// i.e. exactly the sets
//   top    = first k_top entries in the order (value desc, index asc),
//   bottom = first k_bot of the remaining entries in (value asc, index asc).
#pragma once
#include "gear_internal.h"

namespace gear {

// Entry layout a source presents: chunk ch, lane l, slot e  <->  index
// ch*512 + l*8 + e.  src(ch) returns the lane's 8 entries as 16-bit monotone
// KEYS (key16 of the fp16 bit patterns), two per 32-bit word.
//   Src::kMaxChunks > 0 : the vector lives in registers; loops are unrolled.
//   Src::kMaxChunks == 0: runtime loop (vector in LDS).
template <class Src, class F>
__device__ __forceinline__ void for_each_chunk(const Src& src, int nch, F&& f) {
  if constexpr (Src::kMaxChunks > 0) {
#pragma unroll
    for (int ch = 0; ch < Src::kMaxChunks; ++ch)
      if (ch < nch) f(ch, src(ch));
  } else {
    for (int ch = 0; ch < nch; ++ch) f(ch, src(ch));
  }
}

__device__ __forceinline__ uint32_t slot16(const uint4& v, int e) {
  const uint32_t w = (e < 2) ? v.x : (e < 4) ? v.y : (e < 6) ? v.z : v.w;
  return (w >> ((e & 1) * 16)) & 0xFFFFu;
}

// h: 256 counters in LDS (all lanes of the wave see the final values).
// Finds the bin where the count taken from the top reaches k (k >= 1):
// bin, and `above` = entries in bins strictly above it.
__device__ __forceinline__ void scan_from_top(const uint32_t* h, uint32_t k, int& bin, uint32_t& above) {
  const int lane = lane_id();
  uint32_t hh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) hh[i] = h[4 * lane + i];
  const uint32_t s = hh[0] + hh[1] + hh[2] + hh[3];
  const uint32_t suf = wave_incl_suffix(s);
  const unsigned long long m = __ballot(suf >= k);  // lanes 0..L
  const int L = m ? (63 - __clzll((long long)m)) : 0;
  uint32_t cum = suf - s;
  int bsel = 4 * lane;
  uint32_t ab = cum;
  bool done = false;
#pragma unroll
  for (int i = 3; i >= 0; --i) {
    if (!done) {
      if (cum + hh[i] >= k) {
        bsel = 4 * lane + i;
        ab = cum;
        done = true;
      } else {
        cum += hh[i];
      }
    }
  }
  bin = __shfl(bsel, L, 64);
  above = __shfl(ab, L, 64);
}
__device__ __forceinline__ void scan_from_bottom(const uint32_t* h, uint32_t k, int& bin, uint32_t& below) {
  const int lane = lane_id();
  uint32_t hh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) hh[i] = h[4 * lane + i];
  const uint32_t s = hh[0] + hh[1] + hh[2] + hh[3];
  const uint32_t pre = wave_incl_scan(s);
  const unsigned long long m = __ballot(pre >= k);  // lanes L..63
  const int L = m ? (int)__ffsll((long long)m) - 1 : 63;
  uint32_t cum = pre - s;
  int bsel = 4 * lane + 3;
  uint32_t be = cum;
  bool done = false;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (!done) {
      if (cum + hh[i] >= k) {
        bsel = 4 * lane + i;
        be = cum;
        done = true;
      } else {
        cum += hh[i];
      }
    }
  }
  bin = __shfl(bsel, L, 64);
  below = __shfl(be, L, 64);
}

// Index of the m-th (1-based) entry whose key equals tau, in index order.
// No block-level barrier inside (callers branch per wave).
template <class Src>
__device__ __forceinline__ int find_kth_equal(const Src& src, int N, int nch, uint32_t tau, uint32_t m) {
  const int lane = lane_id();
  int found = INT_MAX;
  uint32_t base_cnt = 0;
  bool have = false;
  for_each_chunk(src, nch, [&](int ch, const uint4& v) {
    if (have) return;
    const int base = ch * 512 + lane * 8;
    uint32_t c = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (base + e < N && slot16(v, e) == tau) ++c;
    const uint32_t inc = wave_incl_scan(c);
    const uint32_t total = __shfl(inc, 63, 64);
    if (base_cnt + total >= m) {
      const uint32_t exc = base_cnt + inc - c;
      const bool mine = (exc < m) && (m <= base_cnt + inc);
      int idx = INT_MAX;
      if (mine) {
        uint32_t r = exc;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (base + e < N && slot16(v, e) == tau) {
            ++r;
            if (r == m) idx = base + e;
          }
      }
      const unsigned long long bm = __ballot(mine);
      const int L = bm ? (int)__ffsll((long long)bm) - 1 : 0;
      found = __shfl(idx, L, 64);
      have = true;
    }
    base_cnt += total;
  });
  return found;
}

// A wave with nothing to do passes active = false.  hist: 512 u32 of LDS private to
// the calling wave; only wave-level synchronisation is used, so the waves of a block
// run their selections independently of each other.
template <class Src>
__device__ __forceinline__ Thresh wave_select(const Src& src, int N, int k_top, int k_bot,
                                              uint32_t* hist, bool active) {
  const int lane = lane_id();
  const int nch = active ? ((N + 511) >> 9) : 0;
  Thresh th = thresh_none();

  // ---- level 1: histogram of the high key byte
  for (int i = lane; i < 512; i += 64) hist[i] = 0u;
  wave_lds_sync();
  for_each_chunk(src, nch, [&](int ch, const uint4& v) {
    const int base = ch * 512 + lane * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (base + e < N) atomicAdd(&hist[slot16(v, e) >> 8], 1u);
  });
  wave_lds_sync();
  int bin_t = -1, bin_b = -1;
  uint32_t need_t = 0, need_b = 0;
  if (active && k_top > 0) {
    uint32_t above;
    scan_from_top(hist, (uint32_t)k_top, bin_t, above);
    need_t = (uint32_t)k_top - above;
  }
  if (active && k_bot > 0) {
    uint32_t below;
    scan_from_bottom(hist, (uint32_t)k_bot, bin_b, below);
    need_b = (uint32_t)k_bot - below;
  }
  wave_lds_sync();

  // ---- level 2: histograms of the low key byte inside the two boundary bins
  for (int i = lane; i < 512; i += 64) hist[i] = 0u;
  wave_lds_sync();
  for_each_chunk(src, nch, [&](int ch, const uint4& v) {
    const int base = ch * 512 + lane * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (base + e < N) {
        const uint32_t k = slot16(v, e);
        if ((int)(k >> 8) == bin_t) atomicAdd(&hist[k & 255u], 1u);
        if ((int)(k >> 8) == bin_b) atomicAdd(&hist[256 + (k & 255u)], 1u);
      }
  });
  wave_lds_sync();
  uint32_t need_eq_t = 0, cnt_eq_t = 0, need_eq_b = 0, cnt_eq_b = 0;
  if (active && k_top > 0) {
    int lo;
    uint32_t above;
    scan_from_top(hist, need_t, lo, above);
    th.tau_top = ((uint32_t)bin_t << 8) | (uint32_t)lo;
    need_eq_t = need_t - above;
    cnt_eq_t = hist[lo];
  }
  if (active && k_bot > 0) {
    int lo;
    uint32_t below;
    scan_from_bottom(hist + 256, need_b, lo, below);
    th.tau_bot = ((uint32_t)bin_b << 8) | (uint32_t)lo;
    need_eq_b = need_b - below;
    cnt_eq_b = hist[256 + lo];
  }
  wave_lds_sync();

  // ---- ties: among entries equal to the threshold the lowest indices win;
  // when top and bottom share one threshold value the bottom set continues
  // where the top set stopped.
  if (active && k_top > 0) {
    if (k_bot > 0 && th.tau_top == th.tau_bot) {
      th.i_top = find_kth_equal(src, N, nch, th.tau_top, need_eq_t);
      th.l_bot = th.i_top;
      th.i_bot = (need_eq_t + need_eq_b == cnt_eq_t)
                     ? INT_MAX
                     : find_kth_equal(src, N, nch, th.tau_top, need_eq_t + need_eq_b);
    } else {
      th.i_top = (need_eq_t == cnt_eq_t) ? INT_MAX : find_kth_equal(src, N, nch, th.tau_top, need_eq_t);
      if (k_bot > 0)
        th.i_bot = (need_eq_b == cnt_eq_b) ? INT_MAX : find_kth_equal(src, N, nch, th.tau_bot, need_eq_b);
    }
  }
  return th;
}

}  // namespace gear
