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
//   Src::kMaxChunks < 0 : runtime loop with the loads of several chunks in flight (vector in global memory).
template <class Src, class F>
__device__ __forceinline__ void for_each_chunk(const Src& src, int nch, F&& f) {
  if constexpr (Src::kMaxChunks > 0) {
#pragma unroll
    for (int ch = 0; ch < Src::kMaxChunks; ++ch)
      if (ch < nch) f(ch, src(ch));
  } else if constexpr (Src::kMaxChunks < 0) {
    // vector in global memory: eight chunk loads in flight (reads past the vector return defined data)
    for (int c0 = 0; c0 < nch; c0 += 8) {
      uint4 v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = src(c0 + i);
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (c0 + i < nch) f(c0 + i, v[i]);
    }
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

// The same for both thresholds at once when few entries equal them (the usual case):
// every entry equal to tau_a / tau_b puts its index on a list in LDS (lists[0..63],
// lists[64..127], counters at lists[128], lists[129]); the m-th smallest index of a list
// of at most 64 is then found by ranking.  m_a / m_b = 0: that side is not wanted.
template <class Src>
__device__ __forceinline__ void find_kth_equal_pair(const Src& src, int N, int nch, uint32_t tau_a, uint32_t m_a,
                                                    uint32_t tau_b, uint32_t m_b, uint32_t* lists, int& idx_a,
                                                    int& idx_b) {
  const int lane = lane_id();
  if (lane < 2) lists[128 + lane] = 0u;
  wave_lds_sync();
  const uint32_t ta2 = tau_a | (tau_a << 16), tb2 = tau_b | (tau_b << 16);
  for_each_chunk(src, nch, [&](int ch, const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      // a word with a half equal to tau has a zero half after the xor
      const uint32_t za = w[j] ^ ta2, zb = w[j] ^ tb2;
      const uint32_t hit = (m_a ? ((za - 0x00010001u) & ~za & 0x80008000u) : 0u) |
                           (m_b ? ((zb - 0x00010001u) & ~zb & 0x80008000u) : 0u);
      if (hit) {   // rare
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int idx = ch * 512 + lane * 8 + 2 * j + h;
          const uint32_t k = (w[j] >> (16 * h)) & 0xFFFFu;
          if (idx < N) {
            if (m_a && k == tau_a) {
              const uint32_t pos = atomicAdd(&lists[128], 1u);
              if (pos < 64u) lists[pos] = (uint32_t)idx;
            }
            if (m_b && k == tau_b) {
              const uint32_t pos = atomicAdd(&lists[129], 1u);
              if (pos < 64u) lists[64 + pos] = (uint32_t)idx;
            }
          }
        }
      }
    }
  });
  wave_lds_sync();
  const uint32_t ca = lists[128] < 64u ? lists[128] : 64u, cb = lists[129] < 64u ? lists[129] : 64u;
  const uint32_t mine_a = lane < (int)ca ? lists[lane] : 0xFFFFFFFFu;
  const uint32_t mine_b = lane < (int)cb ? lists[64 + lane] : 0xFFFFFFFFu;
  uint32_t rank_a = 0, rank_b = 0;
  const uint32_t cmax = ca > cb ? ca : cb;
  for (uint32_t j = 0; j < cmax; ++j) {   // wave-uniform trip count
    rank_a += (uint32_t)__shfl(mine_a, (int)j, 64) < mine_a ? 1u : 0u;
    rank_b += (uint32_t)__shfl(mine_b, (int)j, 64) < mine_b ? 1u : 0u;
  }
  idx_a = INT_MAX;
  idx_b = INT_MAX;
  if (m_a) {
    const unsigned long long bm = __ballot(lane < (int)ca && rank_a + 1u == m_a);
    if (bm) idx_a = (int)__shfl(mine_a, (int)__ffsll((long long)bm) - 1, 64);
  }
  if (m_b) {
    const unsigned long long bm = __ballot(lane < (int)cb && rank_b + 1u == m_b);
    if (bm) idx_b = (int)__shfl(mine_b, (int)__ffsll((long long)bm) - 1, 64);
  }
  wave_lds_sync();
}

// Max / min of an unsigned value over each row of 16 lanes, in every lane of the row.
__device__ __forceinline__ uint32_t row16_max_u(uint32_t v) {
  v = max(v, dpp_u<DPP_XOR1>(v));
  v = max(v, dpp_u<DPP_XOR2>(v));
  v = max(v, dpp_u<DPP_HALF_MIRROR>(v));
  v = max(v, dpp_u<DPP_MIRROR>(v));
  return v;
}
__device__ __forceinline__ uint32_t row16_min_u(uint32_t v) {
  v = min(v, dpp_u<DPP_XOR1>(v));
  v = min(v, dpp_u<DPP_XOR2>(v));
  v = min(v, dpp_u<DPP_HALF_MIRROR>(v));
  v = min(v, dpp_u<DPP_MIRROR>(v));
  return v;
}

// Filter_s thresholds of a vector of 128 entries held by one row of 16 lanes, 8 entries per lane
// (entry e of lane oc has in-vector index 8 * oc + e): the per-head Value Filter.  kw: the lane's
// 8 monotone keys, two per word.  The selected sets are the first k_top entries in (value desc,
// index asc) and the first k_bot of the others in (value asc, index asc), found by taking the
// row's largest (smallest) composite below (above) the previous one k_top (k_bot) times; the
// result is the packed predicate of ThreshPair.  All 16 lanes of a row must call together.
__device__ __forceinline__ ThreshPair row16_thresholds(const uint32_t (&kw)[4], int oc, int k_top, int k_bot) {
  uint32_t cT[8], cB[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t k = (e & 1) ? (kw[e >> 1] & 0xFFFF0000u) : (kw[e >> 1] << 16);
    const uint32_t idx = (uint32_t)(8 * oc + e);
    cT[e] = k | (0xFFFFu - idx);
    cB[e] = k | idx;
  }
  ThreshPair p;
  p.top = 0xFFFFFFFFu;   // no composite reaches it: no top outliers
  p.bot = 0u;            // none lies below it: no bottom outliers
  for (int i = 0; i < k_top; ++i) {   // (the counts are the same in every lane)
    uint32_t m = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) m = max(m, cT[e] < p.top ? cT[e] : 0u);
    p.top = row16_max_u(m);
  }
  uint32_t last = 0u;   // composites of finite values are > 0
  for (int i = 0; i < k_bot; ++i) {
    uint32_t m = 0xFFFFFFFFu;
#pragma unroll
    for (int e = 0; e < 8; ++e) m = min(m, (cT[e] < p.top && cB[e] > last) ? cB[e] : 0xFFFFFFFFu);
    last = row16_min_u(m);
  }
  if (k_bot > 0) p.bot = last + 1u;
  return p;
}

constexpr int SELECT_LDS_WORDS = 512;   // LDS words wave_select needs per wave

// A wave with nothing to do passes active = false.  hist: SELECT_LDS_WORDS u32 of LDS private to
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
  // (two copies of the histogram, one for the even and one for the odd lanes: most of a vector falls into a
  // few bins, and adds of one instruction to one address are applied one after another)
  uint32_t* hmine = hist + ((lane & 1) << 8);
  for_each_chunk(src, nch, [&](int ch, const uint4& v) {
    const int base = ch * 512 + lane * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (base + e < N) atomicAdd(&hmine[slot16(v, e) >> 8], 1u);
  });
  wave_lds_sync();
  for (int i = lane; i < 256; i += 64) hist[i] += hist[256 + i];
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
    for (int e = 0; e < 8; ++e) {
      const uint32_t k = slot16(v, e);
      const int hi = (base + e < N) ? (int)(k >> 8) : -2;
      const bool in_t = hi == bin_t, in_b = hi == bin_b;
      // (only the few lanes with an entry in a boundary bin take part: the LDS serves an add of 64 lanes to
      // random bins in ~7 cycles, of a handful of lanes in 2)
      if (in_t || in_b) atomicAdd(&hist[(in_t ? 0u : 256u) + (k & 255u)], 1u);
    }
  });
  wave_lds_sync();
  if (bin_t == bin_b && bin_t >= 0) {   // one bin holds both thresholds: its entries count for both
    for (int i = lane; i < 256; i += 64) hist[256 + i] = hist[i];
    wave_lds_sync();
  }
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
  const bool want_t = active && k_top > 0 && need_eq_t != cnt_eq_t;
  const bool want_b = active && k_bot > 0 && need_eq_b != cnt_eq_b;
  const bool shared = active && k_top > 0 && k_bot > 0 && th.tau_top == th.tau_bot;
  if (!shared && cnt_eq_t <= 64u && cnt_eq_b <= 64u) {
    if (want_t || want_b) {   // wave-uniform
      int it, ib;
      find_kth_equal_pair(src, N, nch, th.tau_top, want_t ? need_eq_t : 0u, th.tau_bot, want_b ? need_eq_b : 0u, hist,
                          it, ib);
      if (want_t) th.i_top = it;
      if (want_b) th.i_bot = ib;
    }
    if (active && k_top > 0 && !want_t) th.i_top = INT_MAX;
    if (active && k_bot > 0 && !want_b) th.i_bot = INT_MAX;
  } else if (active && k_top > 0) {
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
