// Filter_s (Eq. 4) + Quant_b(X - S) (Eq. 2 / Eq. 5) kernels of gear_compress, Key side:
//   k_select_kernel       thresholds of every Key channel vector (over tokens)
//   k_quant_kernel        Key codes, (scale, zero), ordered outlier lists, the filtered input
//                         Y = X - S for the power iteration
// (the Value side is in compress_values.hip)
#include <atomic>
#include "gear_internal.h"
#include "gear_select.h"
#include "gear_launch.h"

namespace gear {

// ------------------------------------------------------------------ sources
struct LdsSource {  // one vector stored contiguously in LDS as 16-bit keys
  static constexpr int kMaxChunks = 0;
  const uint16_t* base;
  int n_pad;  // multiple of 8
  __device__ __forceinline__ uint4 operator()(int ch) const {
    const int off = ch * 512 + lane_id() * 8;
    if (off < n_pad) return *reinterpret_cast<const uint4*>(base + off);
    return make_uint4(0, 0, 0, 0);
  }
};
template <int NC>
struct RegSource {  // the vector lives in the wave's registers
  static constexpr int kMaxChunks = NC;
  const uint4* x;
  __device__ __forceinline__ uint4 operator()(int ch) const { return x[ch]; }
};

// ------------------------------------------------------------------ K select
// 1-D grid of (128/CB) * B*H blocks of 64 * min(CB, 4) threads; LDS: SELECT_LDS_WORDS u32 per wave + [CB][n_pad] keys.
// Consecutive block ids go round-robin to the chip's 8 XCDs (each with its own L2), so
// the id is decoded with the column block fastest INSIDE one XCD: the 128/CB blocks
// that share the 128-byte lines of one slab then meet in one L2 instead of eight.
// CB (channels per block, a power of two) is a template parameter: the row pieces of the
// transposing load are then indexed with shifts and loaded with one fixed instruction.
template <int CB>
__global__ __launch_bounds__(256) void k_select_kernel(const uint16_t* __restrict__ K, int n, int n_pad,
                                                       int nslab, int k_top, int k_bot,
                                                       ThreshPair* __restrict__ thrK, uint32_t* __restrict__ zero,
                                                       int zero_count, uint32_t* __restrict__ ksz, int ng_cap, float qmax) {
  GEAR_DYN_LDS(smem_raw);
  // the first kernel of a compress call also clears the call's list counters (the kernels that
  // count run after this one on the stream)
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < zero_count; i += gridDim.x * blockDim.x) zero[i] = 0u;
  uint32_t* hist_all = reinterpret_cast<uint32_t*>(smem_raw);
  uint16_t* tile = reinterpret_cast<uint16_t*>(smem_raw + (blockDim.x >> 6) * SELECT_LDS_WORDS * sizeof(uint32_t));
  constexpr int ncb = D / CB;
  int slab, cb;
  if ((nslab & 7) == 0) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    cb = j % ncb;
    slab = (j / ncb) * 8 + xcd;
  } else {
    cb = blockIdx.x % ncb;
    slab = blockIdx.x / ncb;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int NT = blockDim.x, NW = NT >> 6;   // 64 threads per vector in flight
  const uint16_t* X = K + (size_t)slab * n * D + cb * CB;

  // transpose-load the [n x CB] column block so every vector is contiguous: a thread takes
  // one row segment (VW channels) of 8 consecutive rows, all 8 loads in flight, turns the
  // values into keys, transposes the 8 x VW block in registers (one byte permute per
  // output word) and stores 8 tokens of a channel with one 16-byte LDS write.  Rows past
  // n get key 0, so stray lanes of the selection read defined data.
  constexpr int VW = CB < 8 ? CB : 8;   // fp16 values per row segment
  constexpr int U = CB / VW;            // row segments per row (a power of two)
  constexpr int NWD = VW >= 2 ? VW / 2 : 1;
  {
    const int ngrp = (n_pad >> 3) * U;
    // a view of the column block that ends with its last row: rows past n read as 0 (the
    // selection never looks at them, they only have to be defined)
    const GEAR_BUF_T xb = GEAR_BUF_MAKE(X, n > 0 ? (n - 1) * (D * 2) + CB * 2 : 0);
    auto load_unit = [&](int gidx, uint32_t (&w)[8][NWD]) {
      const int rg = gidx / U, u = gidx - rg * U;
      const int off = rg * 8 * (D * 2) + u * (VW * 2);
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        if constexpr (VW == 8) {
          const uint4 t4 = GEAR_BUF_LOAD16(xb, off + k * (D * 2));
          w[k][0] = t4.x; w[k][1] = t4.y; w[k][2] = t4.z; w[k][3] = t4.w;
        } else if constexpr (VW == 4) {
          const uint2 t2 = GEAR_BUF_LOAD8(xb, off + k * (D * 2));
          w[k][0] = t2.x; w[k][1] = t2.y;
        } else if constexpr (VW == 2) {
          w[k][0] = GEAR_BUF_LOAD4(xb, off + k * (D * 2));
        } else {
          w[k][0] = GEAR_BUF_LOAD2(xb, off + k * (D * 2));
        }
      }
    };
    auto store_unit = [&](int gidx, uint32_t (&w)[8][NWD]) {
      const int rg = gidx / U, u = gidx - rg * U;
      const int row0 = rg * 8;
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int j = 0; j < NWD; ++j) w[k][j] = key16x2(w[k][j]);
#pragma unroll
      for (int c = 0; c < VW; ++c) {
        const int j = c >> 1;
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;   // the high / the low halves of two words
        const uint4 o = make_uint4(GEAR_BYTE_PERM(w[1][j], w[0][j], sel), GEAR_BYTE_PERM(w[3][j], w[2][j], sel),
                                   GEAR_BYTE_PERM(w[5][j], w[4][j], sel), GEAR_BYTE_PERM(w[7][j], w[6][j], sel));
        *reinterpret_cast<uint4*>(tile + (size_t)(u * VW + c) * n_pad + row0) = o;
      }
    };
    // two units per round, the loads of both in flight together
    for (int gidx = tid; gidx < ngrp; gidx += 2 * NT) {
      uint32_t wa[8][NWD], wb[8][NWD];
      const bool second = gidx + NT < ngrp;
      load_unit(gidx, wa);
      if (second) load_unit(gidx + NT, wb);
      store_unit(gidx, wa);
      if (second) store_unit(gidx + NT, wb);
    }
  }
  block_lds_sync();

  const int iters = (CB + NW - 1) / NW;
  for (int it = 0; it < iters; ++it) {
    const int v = it * NW + wave;
    const bool active = v < CB;
    LdsSource src{tile + (size_t)(active ? v : 0) * n_pad, n_pad};
    const Thresh th = wave_select(src, n, k_top, k_bot, hist_all + wave * SELECT_LDS_WORDS, active);
    if (active && lane == 0) thrK[(size_t)slab * D + cb * CB + v] = pack_thresh(th);
    if (ksz) {
      // per-vector grouping: the channel's one group of this call spans the whole vector, so its
      // (scale, zero) come from here: min and max of X - S, i.e. with the outliers counted as 0
      uint32_t kmn = 0xFFFFu, kmx = 0u;
      if (active) {
        const ThreshPair tp = pack_thresh(th);
        const int nch = (n + 511) >> 9;
        for (int ch = 0; ch < nch; ++ch) {
          const uint4 v4 = src(ch);
          const int base = ch * 512 + lane * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t k = slot16(v4, e), idx = (uint32_t)(base + e);
            if (base + e < n) {
              const bool out = ((k << 16) | (0xFFFFu - idx)) >= tp.top || ((k << 16) | idx) < tp.bot;
              const uint32_t y = out ? 0x8000u : k;
              kmn = min(kmn, y);
              kmx = max(kmx, y);
            }
          }
        }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        kmn = min(kmn, (uint32_t)__shfl_xor(kmn, o, 64));
        kmx = max(kmx, (uint32_t)__shfl_xor(kmx, o, 64));
      }
      if (active && lane == 0)
        ksz[(size_t)slab * ng_cap * D + cb * CB + v] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
    }
  }
}

// ------------------------------------------------------------------ K select, segments of at most 64 tokens
// A flushed buffer: 128 vectors of n_b entries per slab, of which Filter_s keeps one or two.  One block per
// slab, one thread per channel; the slab's rows sit in LDS as keys, row-major as they come, and a thread
// walks down its column.  The selected sets are found by taking the column's largest composite
// (key, index) below the previous one k_top times, then the smallest above the previous one among the
// entries outside the top set k_bot times: (k_top + k_bot) n steps per vector instead of a ranking of
// every entry against every other.  grid (B*H), block 128.
constexpr int KSEL_TINY_ROWS = 64;
__global__ __launch_bounds__(128) void k_select_tiny_kernel(const uint16_t* __restrict__ K, int n, int k_top, int k_bot,
                                                            ThreshPair* __restrict__ thrK, uint32_t* __restrict__ zero,
                                                            int zero_count, uint32_t* __restrict__ ksz, int ng_cap, float qmax) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[KSEL_TINY_ROWS * D];
  // the first kernel of a compress call also clears the call's list counters
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < zero_count; i += gridDim.x * blockDim.x) zero[i] = 0u;
  const int slab = blockIdx.x, c = threadIdx.x;
  {
    const GEAR_BUF_T xb = GEAR_BUF_MAKE(K + (size_t)slab * n * D, n * (D * 2));
    const int npieces = n * (D / 8);   // 16-byte pieces of the slab's rows
    for (int p0 = 0; p0 < npieces; p0 += 4 * 128) {
      uint4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = GEAR_BUF_LOAD16(xb, (p0 + u * 128 + c) * 16);   // pieces past the end read as 0
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int p = p0 + u * 128 + c;
        if (p < npieces)
          *reinterpret_cast<uint4*>(tile + p * 8) = make_uint4(key16x2(v[u].x), key16x2(v[u].y), key16x2(v[u].z), key16x2(v[u].w));
      }
    }
  }
  block_lds_sync();
  Thresh th = thresh_none();
  // composites: (key << 16) | (0xFFFF - index) orders (value desc, index asc) from the top,
  // (key << 16) | index orders (value asc, index asc) from the bottom; all distinct, and the first kind > 0
  uint32_t T = 0u;   // composite of the last top entry
  for (int it = 0; it < k_top; ++it) {
    uint32_t best = 0u;
    for (int j = 0; j < n; ++j) {
      const uint32_t cT = ((uint32_t)tile[j * D + c] << 16) | (0xFFFFu - (uint32_t)j);
      if ((it == 0 || cT < T) && cT > best) best = cT;
    }
    T = best;
  }
  if (k_top > 0 && T != 0u) {
    th.tau_top = T >> 16;
    th.i_top = (int)(0xFFFFu - (T & 0xFFFFu));
  }
  if (k_bot > 0) {
    uint32_t Bc = 0u;
    bool found = true;
    for (int it = 0; it < k_bot && found; ++it) {
      uint32_t best = 0xFFFFFFFFu;
      for (int j = 0; j < n; ++j) {
        const uint32_t key = tile[j * D + c];
        const bool in_top = k_top > 0 && ((key << 16) | (0xFFFFu - (uint32_t)j)) >= T;
        const uint32_t cB = (key << 16) | (uint32_t)j;
        if (!in_top && (it == 0 || cB > Bc) && cB < best) best = cB;
      }
      found = best != 0xFFFFFFFFu;
      Bc = best;
    }
    if (found) {
      th.tau_bot = Bc >> 16;
      th.i_bot = (int)(Bc & 0xFFFFu);
      th.l_bot = (k_top > 0 && th.tau_bot == th.tau_top) ? th.i_top : -1;
    }
  }
  const ThreshPair tp = pack_thresh(th);
  thrK[(size_t)slab * D + c] = tp;
  if (ksz) {
    // per-vector grouping: the channel's one group of this call spans the whole vector: min and max of
    // X - S, i.e. with the outliers counted as 0
    uint32_t kmn = 0xFFFFu, kmx = 0u;
    for (int j = 0; j < n; ++j) {
      const uint32_t k = tile[j * D + c], idx = (uint32_t)j;
      const bool out = ((k << 16) | (0xFFFFu - idx)) >= tp.top || ((k << 16) | idx) < tp.bot;
      const uint32_t y = out ? 0x8000u : k;
      kmn = min(kmn, y);
      kmx = max(kmx, y);
    }
    ksz[(size_t)slab * ng_cap * D + c] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
  }
}

// ------------------------------------------------------------------ K select, segments of more than 8192 tokens
// Such a vector fits neither the registers of a wave nor, eight channels at a time, the LDS of a block, and
// read one channel at a time from the [token][channel] tensor every 2-byte value costs a whole memory
// sector.  So the keys are first written channel-major ([slab][channel][stride] u16, stride = n rounded up
// to 8) into scratch memory, and the selection then reads every vector contiguously, straight from global
// memory, once per pass: no LDS tile, so the occupancy does not depend on the segment length.
struct GlobalKeySource {   // one vector stored contiguously in global memory as 16-bit keys
  static constexpr int kMaxChunks = -1;
  GEAR_BUF_T buf;          // view of the vector's stride keys; reads past it return 0
  __device__ __forceinline__ uint4 operator()(int ch) const { return GEAR_BUF_LOAD16(buf, (ch * 64 + lane_id()) * 16); }
};

// grid (ceil(n / 128), B*H), block 256: thread (rg, oc) takes the 16-byte pieces (8 channels) of rows
// 8 rg .. 8 rg + 7 of the tile, turns the values into keys, transposes the 8 x 8 block in registers and
// stores 8 tokens of each of its 8 channels with one 16-byte store.  Rows past n are written as the key of 0.
__global__ __launch_bounds__(256) void k_transpose_keys_kernel(const uint16_t* __restrict__ K, int n, int stride,
                                                               uint16_t* __restrict__ KT) {
  const int slab = blockIdx.y, tid = threadIdx.x, rg = tid >> 4, oc = tid & 15;
  const int row0 = blockIdx.x * 128 + rg * 8;
  const GEAR_BUF_T xb = GEAR_BUF_MAKE(K + (size_t)slab * n * D, n * (D * 2));
  uint32_t w[8][4];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const uint4 t4 = GEAR_BUF_LOAD16(xb, (row0 + k) * (D * 2) + oc * 16);
    w[k][0] = key16x2(t4.x); w[k][1] = key16x2(t4.y); w[k][2] = key16x2(t4.z); w[k][3] = key16x2(t4.w);
  }
  if (row0 >= stride) return;   // (stride is a multiple of 8: the 8 tokens lie inside or outside together)
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int j = c >> 1;
    const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;   // the high / the low halves of two words
    const uint4 o = make_uint4(GEAR_BYTE_PERM(w[1][j], w[0][j], sel), GEAR_BYTE_PERM(w[3][j], w[2][j], sel),
                               GEAR_BYTE_PERM(w[5][j], w[4][j], sel), GEAR_BYTE_PERM(w[7][j], w[6][j], sel));
    *reinterpret_cast<uint4*>(KT + ((size_t)slab * D + oc * 8 + c) * stride + row0) = o;
  }
}

// grid (B*H * 128 / 4), block 256: one wave per channel vector.
__global__ __launch_bounds__(256) void k_select_long_kernel(const uint16_t* __restrict__ KT, int n, int stride, int k_top,
                                                            int k_bot, ThreshPair* __restrict__ thrK,
                                                            uint32_t* __restrict__ zero, int zero_count,
                                                            uint32_t* __restrict__ ksz, int ng_cap, float qmax) {
  __shared__ uint32_t hist_all[4 * SELECT_LDS_WORDS];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < zero_count; i += gridDim.x * blockDim.x) zero[i] = 0u;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int v = blockIdx.x * 4 + wave;   // slab * 128 + channel
  const GlobalKeySource src{GEAR_BUF_MAKE(KT + (size_t)v * stride, stride * 2)};
  const Thresh th = wave_select(src, n, k_top, k_bot, hist_all + wave * SELECT_LDS_WORDS, true);
  if (lane == 0) thrK[v] = pack_thresh(th);
  if (ksz) {
    // per-vector grouping: (scale, zero) of the channel's one group, from min and max of X - S
    uint32_t kmn = 0xFFFFu, kmx = 0u;
    const ThreshPair tp = pack_thresh(th);
    for_each_chunk(src, (n + 511) >> 9, [&](int ch, const uint4& v4) {
      const int base = ch * 512 + lane * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t k = slot16(v4, e), idx = (uint32_t)(base + e);
        if (base + e < n) {
          const bool out = ((k << 16) | (0xFFFFu - idx)) >= tp.top || ((k << 16) | idx) < tp.bot;
          const uint32_t y = out ? 0x8000u : k;
          kmn = min(kmn, y);
          kmx = max(kmx, y);
        }
      }
    });
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      kmn = min(kmn, (uint32_t)__shfl_xor(kmn, o, 64));
      kmx = max(kmx, (uint32_t)__shfl_xor(kmx, o, 64));
    }
    if (lane == 0)
      ksz[(size_t)(v / D) * ng_cap * D + (v % D)] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
  }
}

// ------------------------------------------------------------------ K select, vectors in registers
// For segments of up to 8192 tokens: a block of eight waves takes eight neighbouring channels, one per
// wave, and every wave ends up with its whole channel vector in registers (NC chunks of 512 keys, the
// layout wave_select reads), so LDS only holds the histograms and a staging buffer and the occupancy no
// longer falls with the segment length.  The vector arrives 1024 tokens at a time: thread tid loads the
// 16-byte row pieces (8 channels) of rows 2 tid and 2 tid + 1, pairs the two rows' keys of each channel
// in one word and writes it to stage[channel][tid]; wave w then reads channel w's 1024 keys back as two
// 16-byte pieces per lane.  All of a thread's loads are requested at the start.
// 1-D grid of 16 * B*H blocks of 512 threads, decoded XCD-aware like k_select_kernel.
template <int NC>
__global__ __launch_bounds__(512, (NC <= 8 ? 4 : 2)) void k_select_reg_kernel(const uint16_t* __restrict__ K, int n, int nslab,
                                                                            int k_top, int k_bot, ThreshPair* __restrict__ thrK,
                                                                            uint32_t* __restrict__ zero, int zero_count,
                                                                            uint32_t* __restrict__ ksz, int ng_cap, float qmax) {
  __shared__ uint32_t hist[8 * SELECT_LDS_WORDS];
  __shared__ __align__(16) uint32_t stage[8][512];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < zero_count; i += gridDim.x * blockDim.x) zero[i] = 0u;
  constexpr int ncb = D / 8;
  int slab, cb;
  if ((nslab & 7) == 0) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    cb = j % ncb;
    slab = (j / ncb) * 8 + xcd;
  } else {
    cb = blockIdx.x % ncb;
    slab = blockIdx.x / ncb;
  }
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // a view of the column block that ends with its last row: rows past n read as 0
  const GEAR_BUF_T xb = GEAR_BUF_MAKE(K + (size_t)slab * n * D + cb * 8, (n - 1) * (D * 2) + 16);
  // every row piece of the thread is requested before the first one is used (rows past n read as 0): the
  // pieces wait in the registers that the finished chunks take over one after another
  uint4 x[NC], raw[NC];
#pragma unroll
  for (int it = 0; it < NC / 2; ++it) {
    raw[2 * it] = GEAR_BUF_LOAD16(xb, (it * 1024 + 2 * tid) * (D * 2));
    raw[2 * it + 1] = GEAR_BUF_LOAD16(xb, (it * 1024 + 2 * tid + 1) * (D * 2));
  }
#pragma unroll
  for (int it = 0; it < NC / 2; ++it) {
    const uint4 ra = raw[2 * it], rb = raw[2 * it + 1];
    const uint32_t ka[4] = {key16x2(ra.x), key16x2(ra.y), key16x2(ra.z), key16x2(ra.w)};
    const uint32_t kb[4] = {key16x2(rb.x), key16x2(rb.y), key16x2(rb.z), key16x2(rb.w)};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      stage[2 * j][tid] = GEAR_BYTE_PERM(kb[j], ka[j], 0x05040100u);       // channel 2j of rows 2 tid, 2 tid + 1
      stage[2 * j + 1][tid] = GEAR_BYTE_PERM(kb[j], ka[j], 0x07060302u);   // channel 2j + 1
    }
    block_lds_sync();
    x[2 * it] = *reinterpret_cast<const uint4*>(&stage[wave][lane * 4]);
    x[2 * it + 1] = *reinterpret_cast<const uint4*>(&stage[wave][256 + lane * 4]);
    block_lds_sync();
  }
  RegSource<NC> src{x};
  const Thresh th = wave_select(src, n, k_top, k_bot, hist + wave * SELECT_LDS_WORDS, true);
  const int ch = cb * 8 + wave;
  if (lane == 0) thrK[(size_t)slab * D + ch] = pack_thresh(th);
  if (ksz) {   // per-vector grouping: the channel's (scale, zero), outliers counted as 0
    const ThreshPair tp = pack_thresh(th);
    uint32_t kmn = 0xFFFFu, kmx = 0u;
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const uint32_t kw[4] = {x[c].x, x[c].y, x[c].z, x[c].w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t k = (e & 1) ? (kw[e >> 1] >> 16) : (kw[e >> 1] & 0xFFFFu), idx = (uint32_t)(c * 512 + lane * 8 + e);
        if ((int)idx < n) {
          const bool out = ((k << 16) | (0xFFFFu - idx)) >= tp.top || ((k << 16) | idx) < tp.bot;
          const uint32_t y = out ? 0x8000u : k;
          kmn = min(kmn, y);
          kmx = max(kmx, y);
        }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      kmn = min(kmn, (uint32_t)__shfl_xor(kmn, o, 64));
      kmx = max(kmx, (uint32_t)__shfl_xor(kmx, o, 64));
    }
    if (lane == 0) ksz[(size_t)slab * ng_cap * D + ch] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
  }
}

// ------------------------------------------------------------------ K quant
// grid (ceil(n/WT), B*H); block 256; WT = max(64, G) tokens per block (G = group size).
// thread (r0 = tid/16, oc = tid%16) owns channels 8*oc..8*oc+7 of rows
// t0 + r0 + 16*k.  The kernel is bound by instruction issue, so the arithmetic is kept
// to what Eq. 2 / Eq. 4 need:
//  * the Filter works on the 16-bit keys, two per word; its result is a mask word
//    (0xFFFF over an outlier's half), which zeroes the entry for min/max and for the
//    quantizer with one bit-select per two entries;
//  * group min / max are taken on the keys (two per instruction) and turned back into
//    fp16 once per (group, channel);
//  * the code goes into its word by a multiply-add (code * 2^(b*e) is exact in fp32);
//  * outlier entries are visited by a loop over the set bits, not over all entries.
template <int G, int BITS>
__global__ __launch_bounds__(256, (G <= 64 ? 3 : 2)) void k_quant_kernel(const uint16_t* __restrict__ K, SegView sv, Dims dm,
                                                      int n, const ThreshPair* __restrict__ thrK,
                                                      uint32_t* __restrict__ pool_ctr,
                                                      uint16_t* __restrict__ Yout) {
  constexpr int WT = G < 64 ? 64 : G;
  constexpr int NK = WT / 16;        // row pieces per thread
  constexpr int NGW = WT / G;        // groups per block (1 or 2)
  constexpr int KPG = NK / NGW;      // row pieces per group
  constexpr float QMAX = (float)((1 << BITS) - 1);
  __shared__ uint32_t red_mn[NGW][4][16][4];   // [group][wave][octet]: 8 keys, two per word
  __shared__ uint32_t red_mx[NGW][4][16][4];
  __shared__ __attribute__((aligned(16))) float gq_mn[NGW][D];
  __shared__ __attribute__((aligned(16))) float gq_inv[NGW][D];
  __shared__ ThreshPair thr_s[D];
  __shared__ uint32_t band_cnt[NK][4];
  __shared__ uint32_t tile_off[2];

  const int slab = blockIdx.y;
  const int t0 = blockIdx.x * WT;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const uint16_t* X = K + (size_t)slab * n * D;

  // every row of the tile is requested before the first one is used
  const GEAR_BUF_T xb = GEAR_BUF_MAKE(X, (uint32_t)n * (D * 2));
  const GEAR_BUF_T yb = GEAR_BUF_MAKE(Yout ? Yout + (size_t)slab * n * D : nullptr, Yout ? (uint32_t)n * (D * 2) : 0u);
  uint32_t raw[NK][4];
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const int t = t0 + r0 + 16 * k;
    const uint4 q = GEAR_BUF_LOAD16(xb, (uint32_t)t * (D * 2) + oc * 16);   // rows past the end read as 0
    raw[k][0] = q.x; raw[k][1] = q.y; raw[k][2] = q.z; raw[k][3] = q.w;
  }
  // thresholds of the 128 channels, staged through LDS: one coalesced read per block
  if (tid < D) thr_s[tid] = dm.ppm > 0 ? thrK[(size_t)slab * D + tid] : pack_thresh(thresh_none());
  block_lds_sync();

  // Filter + group min / max on the keys
  uint32_t msk[NK][4];
  uint32_t mn2[NGW][4], mx2[NGW][4];
#pragma unroll
  for (int gi = 0; gi < NGW; ++gi)
#pragma unroll
    for (int w = 0; w < 4; ++w) { mn2[gi][w] = 0xFFFFFFFFu; mx2[gi][w] = 0u; }
  {
    uint32_t top[8], bot[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { top[e] = thr_s[oc * 8 + e].top; bot[e] = thr_s[oc * 8 + e].bot; }
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int t = t0 + r0 + 16 * k;
#pragma unroll
      for (int w = 0; w < 4; ++w) msk[k][w] = 0u;
      if (t < n) {   // the 16 lanes of a row decide alike
        const uint32_t cT = 0xFFFFu - (uint32_t)t, cB = (uint32_t)t;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t kw = key16x2(raw[k][w]);
          const uint32_t klo = kw << 16, khi = kw & 0xFFFF0000u;
          const bool olo = (klo | cT) >= top[2 * w] || (klo | cB) < bot[2 * w];
          const bool ohi = (khi | cT) >= top[2 * w + 1] || (khi | cB) < bot[2 * w + 1];
          const uint32_t m = (olo ? 0xFFFFu : 0u) | (ohi ? 0xFFFF0000u : 0u);
          msk[k][w] = m;
          const uint32_t yk = (kw & ~m) | (0x80008000u & m);   // an outlier counts as 0 (Eq. 4: X - S)
          mn2[k / KPG][w] = pk_min_u16(mn2[k / KPG][w], yk);
          mx2[k / KPG][w] = pk_max_u16(mx2[k / KPG][w], yk);
        }
      }
    }
  }
  // the four row-threads of a wave that share a channel octet, then the four waves
#pragma unroll
  for (int gi = 0; gi < NGW; ++gi)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      mn2[gi][w] = pk_min_u16(mn2[gi][w], __shfl_xor(mn2[gi][w], 16, 64));
      mn2[gi][w] = pk_min_u16(mn2[gi][w], __shfl_xor(mn2[gi][w], 32, 64));
      mx2[gi][w] = pk_max_u16(mx2[gi][w], __shfl_xor(mx2[gi][w], 16, 64));
      mx2[gi][w] = pk_max_u16(mx2[gi][w], __shfl_xor(mx2[gi][w], 32, 64));
    }
  if (lane < 16) {
#pragma unroll
    for (int gi = 0; gi < NGW; ++gi)
#pragma unroll
      for (int w = 0; w < 4; ++w) { red_mn[gi][wave][oc][w] = mn2[gi][w]; red_mx[gi][wave][oc][w] = mx2[gi][w]; }
  }
  block_lds_sync();
  if (tid < D) {
    const int o = tid >> 3, w = (tid & 7) >> 1, sh = (tid & 1) * 16;
#pragma unroll
    for (int gi = 0; gi < NGW; ++gi) {
      if (t0 + gi * G < n) {
        uint32_t kmn = 0xFFFFu, kmx = 0u;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
          const uint32_t a = (red_mn[gi][wv][o][w] >> sh) & 0xFFFFu, b = (red_mx[gi][wv][o][w] >> sh) & 0xFFFFu;
          kmn = a < kmn ? a : kmn;
          kmx = b > kmx ? b : kmx;
        }
        // per-vector grouping: the channel's one pair of this segment was found with its thresholds
        const GroupQ q = dm.kcvt ? load_group(sv.sz[(size_t)slab * sv.ng_cap * D + tid])
                                 : make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), QMAX);
        gq_mn[gi][tid] = q.mn;
        gq_inv[gi][tid] = q.inv;
        if (!dm.kcvt) sv.sz[((size_t)slab * sv.ng_cap + (t0 + gi * G) / G) * D + tid] = group_bits(q);
      }
    }
  }
  block_lds_sync();

  // codes (packed token-major), and Y = X - S (fp16, outliers zeroed) for the power iteration,
  // which re-derives the quantization error from it
  const GEAR_BUF_T cbuf = GEAR_BUF_MAKE(sv.codes + (size_t)slab * sv.n_cap * dm.wpr, (uint32_t)n * (dm.wpr * 4));
#pragma unroll
  for (int gi = 0; gi < NGW; ++gi) {
    float gmn[8], ginv[8];
    {
      const float4 a0 = *reinterpret_cast<const float4*>(&gq_mn[gi][oc * 8]);
      const float4 a1 = *reinterpret_cast<const float4*>(&gq_mn[gi][oc * 8 + 4]);
      const float4 b0 = *reinterpret_cast<const float4*>(&gq_inv[gi][oc * 8]);
      const float4 b1 = *reinterpret_cast<const float4*>(&gq_inv[gi][oc * 8 + 4]);
      gmn[0] = a0.x; gmn[1] = a0.y; gmn[2] = a0.z; gmn[3] = a0.w; gmn[4] = a1.x; gmn[5] = a1.y; gmn[6] = a1.z; gmn[7] = a1.w;
      ginv[0] = b0.x; ginv[1] = b0.y; ginv[2] = b0.z; ginv[3] = b0.w; ginv[4] = b1.x; ginv[5] = b1.y; ginv[6] = b1.z; ginv[7] = b1.w;
    }
#pragma unroll
    for (int kk = 0; kk < KPG; ++kk) {
      const int k = gi * KPG + kk;
      const int t = t0 + r0 + 16 * k;
      if (t < n) {
#pragma clang fp contract(off)
        float cw0 = 0.0f, cw1 = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t x = raw[k][e >> 1] & ~msk[k][e >> 1];
          const float y = h2f((e & 1) ? (x >> 16) : (x & 0xFFFFu));
          const float tq = __fmul_rn(__fsub_rn(y, gmn[e]), ginv[e]);
          const float c = clamp_f32(rintf(tq), 0.0f, QMAX);
          if (BITS == 2) {
            cw0 = __builtin_fmaf(c, (float)(1u << (2 * e)), cw0);
          } else {
            if (e < 4) cw0 = __builtin_fmaf(c, (float)(1u << (4 * e)), cw0);
            else cw1 = __builtin_fmaf(c, (float)(1u << (4 * (e - 4))), cw1);
          }
        }
        // (an empty view when the caller wants no Y)
        GEAR_BUF_STORE16_NT(yb, (uint32_t)t * (D * 2) + oc * 16,
                            make_uint4(raw[k][0] & ~msk[k][0], raw[k][1] & ~msk[k][1], raw[k][2] & ~msk[k][2], raw[k][3] & ~msk[k][3]));
        if (BITS == 4) {
          GEAR_BUF_STORE4(cbuf, (uint32_t)t * (dm.wpr * 4) + oc * 4, (uint32_t)cw0 | ((uint32_t)cw1 << 16));
        } else {  // 2 bits: 16 bits per thread
          GEAR_BUF_STORE2(cbuf, (uint32_t)t * (dm.wpr * 4) + oc * 2, (uint32_t)cw0);
        }
      }
    }
  }

  // Outliers of a token row: the first ELL_K in channel order take the row's fixed
  // slots, the rest go to the tile's overflow list, ordered (t, c).  The 16 lanes
  // that own a row are 16 consecutive lanes.
  if (dm.ppm > 0) {
    uint32_t fl8[NK];                      // bit e: entry e of the row piece is an outlier
    uint32_t cnt[NK], inc[NK], pre[NK];    // overflow entries of this lane, their scan over the wave; outliers of the row before this lane
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int t = t0 + r0 + 16 * k;
      uint32_t f = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t x = msk[k][w] & 0x00010001u;
        f |= ((x | (x >> 15)) & 3u) << (2 * w);
      }
      fl8[k] = f;
      const uint32_t c_all = __popc(f);
      uint32_t rinc = c_all;              // inclusive scan over the row's 16 lanes
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) {
        const uint32_t up = __shfl_up(rinc, o, 16);
        if (oc >= o) rinc += up;
      }
      pre[k] = rinc - c_all;
      const uint32_t row_total = __shfl(rinc, 15, 16);
      const uint32_t in_slots = pre[k] >= ELL_K ? 0u : (pre[k] + c_all > ELL_K ? ELL_K - pre[k] : c_all);
      cnt[k] = c_all - in_slots;
      if (t < n) {
        uint32_t* slots = sv.ell + ((size_t)slab * sv.n_cap + t) * ELL_K;
        uint32_t s_i = pre[k], ff = f;
        while (ff != 0u && s_i < ELL_K) {
          const int e = __ffs((int)ff) - 1;
          ff &= ff - 1u;
          slots[s_i] = (uint32_t)(oc * 8 + e) | ELL_VALID | (half_of(raw[k][0], raw[k][1], raw[k][2], raw[k][3], e) << 16);
          ++s_i;
        }
        if (oc < ELL_K && (uint32_t)oc >= row_total) slots[oc] = 0u;   // empty slots
      }
      // rows with more than ELL_K outliers are the exception: most waves have nothing to scan
      inc[k] = __ballot(cnt[k] != 0u) != 0ull ? wave_incl_scan(cnt[k]) : 0u;
      if (lane == 63) band_cnt[k][wave] = inc[k];
    }
    block_lds_sync();
    if (tid < WT / TILE) {
      uint32_t tot = 0;
      for (int k = tid * 4; k < tid * 4 + 4; ++k)
        for (int w = 0; w < 4; ++w) tot += band_cnt[k][w];
      const int tile = t0 / TILE + tid;
      uint32_t off = 0;
      if (t0 + tid * TILE < n) {
        off = atomicAdd(&pool_ctr[slab], tot);
        sv.sp_table[(size_t)slab * sv.ntile_cap + tile] = make_uint2(off, tot);
      }
      tile_off[tid] = off;
    }
    block_lds_sync();
    uint32_t* pool = sv.sp_pool + (size_t)slab * sv.pool_cap;
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      if (cnt[k] == 0u) continue;          // rows with more than ELL_K outliers are the exception
      const int tl = r0 + 16 * k;
      const int ti = k / 4;  // tile inside the block
      uint32_t off = tile_off[ti];
      for (int kk = ti * 4; kk < k; ++kk)
        for (int w = 0; w < 4; ++w) off += band_cnt[kk][w];
      for (int w = 0; w < wave; ++w) off += band_cnt[k][w];
      off += inc[k] - cnt[k];
      uint32_t s_i = pre[k], ff = fl8[k];
      while (ff != 0u) {
        const int e = __ffs((int)ff) - 1;
        ff &= ff - 1u;
        if (s_i >= ELL_K) {
          if (off < sv.pool_cap) pool[off] = (uint32_t)((tl & 63) * D + oc * 8 + e) | (half_of(raw[k][0], raw[k][1], raw[k][2], raw[k][3], e) << 16);
          ++off;
        }
        ++s_i;
      }
    }
  }
}

// ------------------------------------------------------------------ launchers
constexpr size_t KSEL_TILE_BYTES = 32768;   // LDS tile of one block: 4 blocks per CU; smaller tiles mean 4-byte row pieces, measured slower
static int k_select_cb(int n_pad, int slabs) {
  int cb = 128;
  while (cb > 1 && (size_t)cb * n_pad * 2 > KSEL_TILE_BYTES) cb >>= 1;
  // short segments (a flushed buffer): more, smaller blocks, so that the vectors are selected
  // side by side instead of 32 after another in each wave
  while (cb > 4 && (128 / cb) * slabs < 4096) cb >>= 1;
  return cb;
}

template <int CB>
static hipError_t launch_k_select_cb(const uint16_t* K, const Dims& dm, int n, int n_pad, int k_top, int k_bot,
                                     ThreshPair* thrK, uint32_t* zero, int zero_count, const SegView& sv, hipStream_t st) {
  constexpr int nw = CB < 4 ? CB : 4;   // waves per block: one vector each per round
  const size_t lds = (size_t)nw * SELECT_LDS_WORDS * sizeof(uint32_t) + (size_t)CB * n_pad * 2;
  static std::atomic<size_t> lds_allowed{0};   // per kernel instance (CB): raised when a launch needs more than any before
  if (lds > lds_allowed.load(std::memory_order_relaxed)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_select_kernel<CB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_allowed.store(lds, std::memory_order_relaxed);
  }
  dim3 grid((D / CB) * dm.B * dm.H);
  hipLaunchKernelGGL(k_select_kernel<CB>, grid, dim3(64 * nw), lds, st, K, n, n_pad, dm.B * dm.H, k_top, k_bot, thrK, zero,
                     zero_count, dm.kcvt ? sv.sz : (uint32_t*)nullptr, sv.ng_cap, dm.qmax);
  return hipGetLastError();
}

template <int NC>
static hipError_t launch_k_select_reg(const uint16_t* K, const Dims& dm, int n, int k_top, int k_bot, ThreshPair* thrK,
                                      uint32_t* zero, int zero_count, const SegView& sv, hipStream_t st) {
  hipLaunchKernelGGL(k_select_reg_kernel<NC>, dim3((D / 8) * dm.B * dm.H), dim3(512), 0, st, K, n, dm.B * dm.H, k_top, k_bot, thrK,
                     zero, zero_count, dm.kcvt ? sv.sz : (uint32_t*)nullptr, sv.ng_cap, dm.qmax);
  return hipGetLastError();
}

hipError_t launch_k_select(const uint16_t* K, const Dims& dm, int n, int k_top, int k_bot, ThreshPair* thrK,
                           uint32_t* zero, int zero_count, const SegView& sv, uint16_t* kt_scratch, hipStream_t st) {
  // segments of more than 8192 tokens: through a channel-major copy of the keys
  if (n > 8192 && kt_scratch != nullptr) {
    const int stride = (n + 7) & ~7;
    hipLaunchKernelGGL(k_transpose_keys_kernel, dim3((n + 127) / 128, dm.B * dm.H), dim3(256), 0, st, K, n, stride, kt_scratch);
    hipLaunchKernelGGL(k_select_long_kernel, dim3(dm.B * dm.H * (D / 4)), dim3(256), 0, st, (const uint16_t*)kt_scratch, n,
                       stride, k_top, k_bot, thrK, zero, zero_count, dm.kcvt ? sv.sz : (uint32_t*)nullptr, sv.ng_cap, dm.qmax);
    return hipGetLastError();
  }
  // a flushed buffer: one thread per channel vector
  if (n <= KSEL_TINY_ROWS) {
    hipLaunchKernelGGL(k_select_tiny_kernel, dim3(dm.B * dm.H), dim3(128), 0, st, K, n, k_top, k_bot, thrK, zero, zero_count,
                       dm.kcvt ? sv.sz : (uint32_t*)nullptr, sv.ng_cap, dm.qmax);
    return hipGetLastError();
  }
  // segments of 1025 .. 8192 tokens: the channel vectors live in registers
  if (n > 4096 && n <= 8192) return launch_k_select_reg<16>(K, dm, n, k_top, k_bot, thrK, zero, zero_count, sv, st);
  if (n > 2048 && n <= 4096) return launch_k_select_reg<8>(K, dm, n, k_top, k_bot, thrK, zero, zero_count, sv, st);
  if (n > 1024 && n <= 2048) return launch_k_select_reg<4>(K, dm, n, k_top, k_bot, thrK, zero, zero_count, sv, st);
  const int n_pad = (n + 7) & ~7;
  switch (k_select_cb(n_pad, dm.B * dm.H)) {
    case 128: return launch_k_select_cb<128>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 64: return launch_k_select_cb<64>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 32: return launch_k_select_cb<32>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 16: return launch_k_select_cb<16>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 8: return launch_k_select_cb<8>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 4: return launch_k_select_cb<4>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    case 2: return launch_k_select_cb<2>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
    default: return launch_k_select_cb<1>(K, dm, n, n_pad, k_top, k_bot, thrK, zero, zero_count, sv, st);
  }
}

template <int G>
static void launch_k_quant_g(const uint16_t* K, const SegView& sv, const Dims& dm, int n, const ThreshPair* thrK,
                             uint32_t* pool_ctr, uint16_t* Yout, hipStream_t st) {
  constexpr int WT = G < 64 ? 64 : G;
  dim3 grid((n + WT - 1) / WT, dm.B * dm.H);
  if (dm.bits == 2)
    hipLaunchKernelGGL((k_quant_kernel<G, 2>), grid, dim3(256), 0, st, K, sv, dm, n, thrK, pool_ctr, Yout);
  else
    hipLaunchKernelGGL((k_quant_kernel<G, 4>), grid, dim3(256), 0, st, K, sv, dm, n, thrK, pool_ctr, Yout);
}

hipError_t launch_k_quant(const uint16_t* K, const SegView& sv, const Dims& dm, int n, const ThreshPair* thrK,
                          uint32_t* pool_ctr, uint16_t* Yout, hipStream_t st) {
  if (dm.g == 128) launch_k_quant_g<128>(K, sv, dm, n, thrK, pool_ctr, Yout, st);
  else if (dm.g == 64) launch_k_quant_g<64>(K, sv, dm, n, thrK, pool_ctr, Yout, st);
  else launch_k_quant_g<32>(K, sv, dm, n, thrK, pool_ctr, Yout, st);
  return hipGetLastError();
}

}  // namespace gear
