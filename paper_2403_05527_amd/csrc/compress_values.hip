// Filter_s (Eq. 4) + Quant_b(X - S) (Eq. 2 / Eq. 5) kernels of gear_compress, Value side:
//   v_select_kernel  thresholds of every Value token vector: the token's row over
//                    ALL heads' channels (index j = h*128 + c), one wave per token
//                    with the vector in registers
//   v_quant_kernel   per (b, h, 64-token tile): outlier predicate, per-token group
//                    min/max inside the row (lane exchanges), codes written in the
//                    token-blocked order the decode kernel's MFMA operand expects,
//                    (scale, zero), the tile's outlier list ordered (c, t), the filtered
//                    input Y = X - S for the power iteration
#include "gear_internal.h"
#include "gear_select.h"
#include "gear_select_rows.h"
#include "gear_launch.h"

namespace gear {

template <int NC>
struct RegSource {  // the vector lives in the wave's registers
  static constexpr int kMaxChunks = NC;
  const uint4* x;
  __device__ __forceinline__ uint4 operator()(int ch) const { return x[ch]; }
};

// grid (ceil(n / (4 * tpw)), B); block 256: tpw tokens per wave, one after another.
// lane l, chunk ch  <->  head 4*ch + l/16, channels 8*(l%16)..+7, i.e. in-vector index
// ch*512 + l*8 + e.
// Under the per-vector grouping (vsz != nullptr) the kernel also leaves the token's (scale, zero):
// its one Value group spans the whole vector, outliers counted as 0.  per_head: the Filter ranks
// each head's 128 channels (the 16 lanes of a row) on their own; thresholds are then not stored
// (the quantization kernel finds them again, they cost less than their round trip).
template <int NC>
__global__ __launch_bounds__(256, (NC <= 8 ? 5 : NC <= 10 ? 4 : 2)) void v_select_kernel(const uint16_t* __restrict__ V, int H, int n, int tpw, int k_top,
                                                       int k_bot, ThreshPair* __restrict__ thrV, uint32_t* __restrict__ vsz,
                                                       float qmax, int per_head) {
  __shared__ uint32_t hist[4 * SELECT_LDS_WORDS];
  const int b = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hsub = lane >> 4, oc = lane & 15;
  const int N = H * D;
  for (int i = 0; i < tpw; ++i) {
    const int t = (blockIdx.x * tpw + i) * 4 + wave;
    const bool tvalid = t < n;
    // (a view of the batch element's H * n rows: heads past H read as 0; entries past N are
    // never looked at by the selection, they only have to be defined)
    const GEAR_BUF_T vb = GEAR_BUF_MAKE(V + (size_t)b * H * n * D, tvalid ? (uint32_t)H * n * (D * 2) : 0u);
    const uint32_t off0 = ((uint32_t)hsub * n + t) * (D * 2) + oc * 16;
    uint4 x[NC];
#pragma unroll
    for (int ch = 0; ch < NC; ++ch) {
      const uint4 raw = GEAR_BUF_LOAD16(vb, off0 + (uint32_t)ch * 4u * n * (D * 2));
      x[ch] = make_uint4(key16x2(raw.x), key16x2(raw.y), key16x2(raw.z), key16x2(raw.w));
    }
    ThreshPair tp = pack_thresh(thresh_none());
    if (!per_head) {
      RegSource<NC> src{x};
      const Thresh th = wave_select(src, N, k_top, k_bot, hist + wave * SELECT_LDS_WORDS, tvalid);
      tp = pack_thresh(th);
      if (tvalid && lane == 0 && thrV) thrV[(size_t)b * n + t] = tp;
    }
    if (vsz) {
      uint32_t kmn = 0xFFFFu, kmx = 0u;
#pragma unroll
      for (int ch = 0; ch < NC; ++ch) {
        const uint32_t kw[4] = {x[ch].x, x[ch].y, x[ch].z, x[ch].w};
        uint32_t idx0 = (uint32_t)(ch * 512 + lane * 8);          // index in the token's row over all heads
        if (per_head) {
          tp = row16_thresholds(kw, oc, k_top, k_bot);            // this head's own thresholds,
          idx0 = (uint32_t)(oc * 8);                              // on the index inside the head
        }
        if (ch * 512 + lane * 8 < N) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t k = (e & 1) ? (kw[e >> 1] >> 16) : (kw[e >> 1] & 0xFFFFu), idx = idx0 + e;
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
      if (tvalid && lane == 0) vsz[(size_t)b * n + t] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
    }
  }
}

// The same thresholds for token rows of at most 1024 entries (up to eight KV heads), four tokens per
// wave: row r of 16 lanes takes token 4 (4 (blockIdx.x tpw + it) + wave) + r, lane i of the row the
// 16-byte piece i (channels 8 i .. 8 i + 7) of each head (gear_select_rows.h).  grid (ceil(n / (16 tpw)), B),
// block 256, 2 KB of LDS per row.  vsz: nullptr unless the per-vector grouping is on.
__global__ __launch_bounds__(256, 4) void v_select_rows_kernel(const uint16_t* __restrict__ V, int H, int n, int tpw,
                                                               int k_top, int k_bot, ThreshPair* __restrict__ thrV,
                                                               uint32_t* __restrict__ vsz, float qmax) {
  __shared__ __attribute__((aligned(16))) uint32_t hist[16 * SELECT_ROW_LDS_WORDS];
  const int b = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, row = lane >> 4, i = lane & 15;
  uint32_t* hrow = hist + (wave * 4 + row) * SELECT_ROW_LDS_WORDS;
  // a view of the batch element's H * n rows; a lane whose token does not exist reads past it (zeros)
  const GEAR_BUF_T vb = GEAR_BUF_MAKE(V + (size_t)b * H * n * D, (uint32_t)H * n * (D * 2));
  for (int it = 0; it < tpw; ++it) {
    const int t = ((blockIdx.x * tpw + it) * 4 + wave) * 4 + row;
    const bool tvalid = t < n;
    const uint32_t off0 = tvalid ? (uint32_t)t * (D * 2) + i * 16 : 0xFFFFFF00u;
    uint4 x[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) {
      x[h] = make_uint4(0, 0, 0, 0);
      if (h < H) {
        const uint4 raw = GEAR_BUF_LOAD16(vb, tvalid ? off0 + (uint32_t)h * n * (D * 2) : off0);
        x[h] = make_uint4(key16x2(raw.x), key16x2(raw.y), key16x2(raw.z), key16x2(raw.w));
      }
    }
    ThreshPair tp = pack_thresh(thresh_none());
    if (k_top > 0 || k_bot > 0) {
      tp = pack_thresh(row_select(x, H, k_top, k_bot, hrow));
      if (tvalid && i == 0 && thrV) thrV[(size_t)b * n + t] = tp;
    }
    if (vsz) {   // per-vector grouping: the token's (scale, zero), outliers counted as 0
      uint32_t kmn = 0xFFFFu, kmx = 0u;
#pragma unroll
      for (int h = 0; h < 8; ++h)
        if (h < H) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const uint32_t k = slot16(x[h], e), idx = (uint32_t)(128 * h + 8 * i + e);
            const bool out = ((k << 16) | (0xFFFFu - idx)) >= tp.top || ((k << 16) | idx) < tp.bot;
            const uint32_t y = out ? 0x8000u : k;
            kmn = min(kmn, y);
            kmx = max(kmx, y);
          }
        }
      kmn = row16_min_u(kmn);
      kmx = row16_max_u(kmx);
      if (tvalid && i == 0) vsz[(size_t)b * n + t] = group_bits(make_group(h2f(unkey16(kmn)), h2f(unkey16(kmx)), qmax));
    }
  }
}

// grid (ceil(n/64), B*H); block 256; thread (r0 = tid/16, oc = tid%16) owns
// channels 8*oc..+7 of rows t0 + r0 + 16*k, k = 0..3.  Same arithmetic as the Key
// kernel: Filter and min/max on packed 16-bit keys with a mask word per two entries,
// code bytes read off float mantissas.
template <int BITS>
__global__ __launch_bounds__(256) void v_quant_kernel(const uint16_t* __restrict__ V, SegView sv, Dims dm, int n,
                                                      const ThreshPair* __restrict__ thrV, const uint32_t* __restrict__ vsz,
                                                      int k_top, int k_bot, uint32_t* __restrict__ pool_ctr,
                                                      uint16_t* __restrict__ Yout) {
  constexpr int PITCH = 136;  // bytes per staged code row (multiple of 8)
  constexpr float QMAX = (float)((1 << BITS) - 1);
  constexpr int bits = BITS, tpw = 32 / BITS;
  __shared__ __align__(16) uint8_t stage[TILE * PITCH];
  __shared__ uint32_t colmask[D][2];
  __shared__ uint16_t oval[D][TILE + 2];   // fp16 values of the tile's outliers (only their cells are written)
  __shared__ uint32_t wtot[2];
  __shared__ uint32_t list_off;
  const int slab = blockIdx.y, tile = blockIdx.x;
  const int b = slab / dm.H, h = slab - b * dm.H;
  const int t0 = tile * TILE;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const int g = dm.g, lg = 31 - __clz(g);   // g is a power of two
  const uint16_t* X = V + (size_t)slab * n * D;

  if (tid < D) { colmask[tid][0] = 0u; colmask[tid][1] = 0u; }
  block_lds_sync();

  // every row of the tile and its thresholds are requested before the first one is used
  const GEAR_BUF_T xb = GEAR_BUF_MAKE(X, (uint32_t)n * (D * 2));
  const GEAR_BUF_T yb = GEAR_BUF_MAKE(Yout ? Yout + (size_t)slab * n * D : nullptr, Yout ? (uint32_t)n * (D * 2) : 0u);
  uint4 xrow[4];
  ThreshPair trow[4];
  uint32_t gsz[4];   // per-vector grouping: the token's (scale, zero)
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int t = t0 + r0 + 16 * k;
    xrow[k] = GEAR_BUF_LOAD16(xb, (uint32_t)t * (D * 2) + oc * 16);   // rows past the end read as 0
    trow[k] = pack_thresh(thresh_none());                             // and have no outliers
    if (t < n && dm.ppm > 0 && !dm.vhead) trow[k] = thrV[(size_t)b * n + t];
    gsz[k] = 0u;
    if (t < n && dm.kcvt) gsz[k] = vsz[(size_t)b * n + t];
  }
  if (dm.vhead && dm.ppm > 0) {   // the Filter per head: the row's 16 lanes hold the whole vector
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t kw[4] = {key16x2(xrow[k].x), key16x2(xrow[k].y), key16x2(xrow[k].z), key16x2(xrow[k].w)};
      const ThreshPair tp = row16_thresholds(kw, oc, k_top, k_bot);
      if (t0 + r0 + 16 * k < n) trow[k] = tp;
    }
  }
  // in-vector index of entry e: h*128 + 8*oc + e (8*oc + e when the Filter is per head); the low three bits are e
  const uint32_t cB0 = (uint32_t)((dm.vhead ? 0 : h * D) + oc * 8), cT0 = (0xFFFFu - cB0) & ~7u;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int tl = r0 + 16 * k, t = t0 + tl;
    const bool tv = t < n;
    const uint32_t raw[4] = {xrow[k].x, xrow[k].y, xrow[k].z, xrow[k].w};
    const uint32_t top = trow[k].top, bot = trow[k].bot;
    uint32_t msk[4];
    uint32_t mn2 = 0xFFFFFFFFu, mx2 = 0u;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t kw = key16x2(raw[w]);
      const uint32_t klo = kw << 16, khi = kw & 0xFFFF0000u;
      const bool olo = (klo | cT0 | (uint32_t)(7 - 2 * w)) >= top || (klo | cB0 | (uint32_t)(2 * w)) < bot;
      const bool ohi = (khi | cT0 | (uint32_t)(6 - 2 * w)) >= top || (khi | cB0 | (uint32_t)(2 * w + 1)) < bot;
      const uint32_t m = (olo ? 0xFFFFu : 0u) | (ohi ? 0xFFFF0000u : 0u);
      msk[w] = m;
      const uint32_t yk = (kw & ~m) | (0x80008000u & m);   // an outlier counts as 0 (Eq. 4: X - S)
      mn2 = pk_min_u16(mn2, yk);
      mx2 = pk_max_u16(mx2, yk);
    }
    // column bitmask of the tile's outliers (few entries: visited by set bit)
    {
      uint32_t f = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t x = msk[w] & 0x00010001u;
        f |= ((x | (x >> 15)) & 3u) << (2 * w);
      }
      while (f != 0u) {
        const int e = __ffs((int)f) - 1;
        f &= f - 1u;
        atomicOr(&colmask[oc * 8 + e][tl >> 5], 1u << (tl & 31));
        oval[oc * 8 + e][tl] = (uint16_t)half_of(raw[0], raw[1], raw[2], raw[3], e);
      }
    }
    // group = g consecutive channels of the row = g/8 neighbouring lanes
    // (reduced as integer keys: the lane exchange folds into the min / max instruction)
    uint32_t kmn = mn2 & 0xFFFFu, kmx = mx2 & 0xFFFFu;
    kmn = min(kmn, mn2 >> 16);
    kmx = max(kmx, mx2 >> 16);
    kmn = min(kmn, dpp_u<DPP_XOR1>(kmn));
    kmx = max(kmx, dpp_u<DPP_XOR1>(kmx));
    kmn = min(kmn, dpp_u<DPP_XOR2>(kmn));
    kmx = max(kmx, dpp_u<DPP_XOR2>(kmx));
    if (g >= 64) {
      kmn = min(kmn, dpp_u<DPP_HALF_MIRROR>(kmn));
      kmx = max(kmx, dpp_u<DPP_HALF_MIRROR>(kmx));
    }
    if (g >= 128) {
      kmn = min(kmn, dpp_u<DPP_MIRROR>(kmn));
      kmx = max(kmx, dpp_u<DPP_MIRROR>(kmx));
    }
    const float lmn = h2f(unkey16(kmn)), lmx = h2f(unkey16(kmx));
    const GroupQ q = dm.kcvt ? load_group(gsz[k]) : make_group(lmn, lmx, QMAX);
    uint32_t fc[8];   // bits of code + 2^23
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma clang fp contract(off)
      const uint32_t x = raw[e >> 1] & ~msk[e >> 1];
      const float y = h2f((e & 1) ? (x >> 16) : (x & 0xFFFFu));
      const float tq = __fmul_rn(__fsub_rn(y, q.mn), q.inv);
      const float c = clamp_f32(rintf(tq), 0.0f, QMAX);
      fc[e] = __float_as_uint(c + 8388608.0f);   // low byte of the mantissa = the code
    }
    // 8 code bytes (0 for a row past the end)
    const uint32_t cb0 = tv ? low_bytes4(fc[0], fc[1], fc[2], fc[3]) : 0u;
    const uint32_t cb1 = tv ? low_bytes4(fc[4], fc[5], fc[6], fc[7]) : 0u;
    *reinterpret_cast<uint2*>(&stage[tl * PITCH + oc * 8]) = make_uint2(cb0, cb1);
    if (tv) {
      if ((oc & ((g >> 3) - 1)) == 0) sv.sz[((size_t)slab * sv.n_cap + t) * (D >> lg) + ((oc * 8) >> lg)] = group_bits(q);
    }
    // Y = X - S (fp16, outliers zeroed): the power iteration re-derives the quantization error from it
    // (an empty view when the caller wants no Y; rows past the end fall outside the view)
    GEAR_BUF_STORE16_NT(yb, (uint32_t)t * (D * 2) + oc * 16,
                        make_uint4(raw[0] & ~msk[0], raw[1] & ~msk[1], raw[2] & ~msk[2], raw[3] & ~msk[3]));
  }
  block_lds_sync();

  // code words in operand order: block of 4*tpw tokens, word (kg*16 + c%16)*8 + c/16 holds
  // channel c for tokens tpw*kg + i at bits i*b
  {
    const int TB = 4 * tpw;               // tokens per block: 64 (2 bits) or 32 (4 bits)
    const int nblk = TILE / TB;           // blocks in this tile
    for (int d = tid; d < nblk * 512; d += 256) {
      const int blk = d >> 9, rem = d & 511;
      const int kg = rem >> 7, n16 = (rem >> 3) & 15, j = rem & 7;
      const int c = 16 * j + n16;
      const int row0 = blk * TB + kg * tpw;
      // every word of a block that holds at least one token is written (rows past n carry code 0),
      // so a reader of the block never sees stale memory
      if (t0 + blk * TB < n) {
        uint32_t word = 0;
        for (int i = 0; i < tpw; ++i) word |= (uint32_t)stage[(row0 + i) * PITCH + c] << (i * bits);
        sv.codes[((size_t)slab * sv.nblk_cap + (size_t)tile * nblk + blk) * 512 + rem] = word;
      }
    }
  }

  // Outliers of this (head, tile): thread c owns channel c.  The first ELL_V of a
  // channel in token order take the channel's fixed slots, the rest go to the tile's
  // overflow list, ordered (c, t).
  if (dm.ppm > 0) {
    uint32_t m0 = 0, m1 = 0, cnt = 0, inc = 0;
    if (tid < D) {
      m0 = colmask[tid][0];
      m1 = colmask[tid][1];
      const uint32_t c_all = __popc(m0) + __popc(m1);
      cnt = c_all > ELL_V ? c_all - ELL_V : 0u;
    }
    if (wave < 2) {
      inc = wave_incl_scan(cnt);
      if (lane == 63) wtot[wave] = inc;
    }
    block_lds_sync();
    if (tid == 0) {
      const uint32_t tot = wtot[0] + wtot[1];
      // a list that fits takes the tile's reserved region; a longer one is allocated behind the regions
      const uint32_t off = tot <= VPOOL_FIXED ? (uint32_t)(h * sv.ntile_cap + tile) * VPOOL_FIXED
                                              : (uint32_t)(dm.H * sv.ntile_cap) * VPOOL_FIXED + atomicAdd(&pool_ctr[b], tot);
      sv.sp_table[(size_t)slab * sv.ntile_cap + tile] = make_uint2(off, tot);
      list_off = off;
    }
    block_lds_sync();
    if (tid < D) {
      uint32_t off = list_off + (wave == 1 ? wtot[0] : 0u) + inc - cnt;
      uint32_t* pool = sv.sp_pool + (size_t)b * sv.pool_cap;
      uint32_t slot[ELL_V];
#pragma unroll
      for (int i = 0; i < ELL_V; ++i) slot[i] = 0u;   // empty slots
      uint32_t s_i = 0;
      for (int half = 0; half < 2; ++half) {
        uint32_t mm = half ? m1 : m0;
        while (mm) {
          const int bit = __ffs((int)mm) - 1;
          mm &= mm - 1;
          const int tl = half * 32 + bit;
          const uint32_t hb = oval[tid][tl];
          if (s_i < ELL_V) {
#pragma unroll
            for (int i = 0; i < ELL_V; ++i)
              if (s_i == (uint32_t)i) slot[i] = (uint32_t)tl | ELL_VALID | (hb << 16);
          } else {
            if (off < sv.pool_cap) pool[off] = (uint32_t)(tl * D + tid) | (hb << 16);
            ++off;
          }
          ++s_i;
        }
      }
      static_assert(ELL_V == 2, "the channel's slots are stored as one 8-byte word");
      *reinterpret_cast<uint2*>(sv.ell + (((size_t)slab * sv.ntile_cap + tile) * D + tid) * ELL_V) = make_uint2(slot[0], slot[1]);
    }
  }
}

// ------------------------------------------------------------------ launchers
template <int NC>
static hipError_t launch_vsel(const uint16_t* V, const Dims& dm, int n, int k_top, int k_bot, ThreshPair* thrV, uint32_t* vsz,
                              hipStream_t st) {
  // four tokens per wave, or one when the call has few tokens (a flushed buffer)
  const int tpw = (long long)n * dm.B >= 16384 ? 4 : 1;
  dim3 grid((n + 4 * tpw - 1) / (4 * tpw), dm.B);
  hipLaunchKernelGGL(v_select_kernel<NC>, grid, dim3(256), 0, st, V, dm.H, n, tpw, k_top, k_bot, thrV,
                     dm.kcvt ? vsz : (uint32_t*)nullptr, dm.qmax, dm.vhead);
  return hipGetLastError();
}

hipError_t launch_v_filter_quant(const uint16_t* V, const SegView& sv, const Dims& dm, int n, int k_top,
                                 int k_bot, ThreshPair* thrV, uint32_t* vsz, uint32_t* pool_ctr, uint16_t* Yout,
                                 hipStream_t st) {
  // the pass over whole token rows: thresholds of the per-token Filter, and a token's (scale, zero)
  // under the per-vector grouping
  if ((dm.ppm > 0 && !dm.vhead) || dm.kcvt) {
    const int kt = dm.ppm > 0 ? k_top : 0, kb = dm.ppm > 0 ? k_bot : 0;
    const int nc = (dm.H + 3) / 4;
    hipError_t e;
    const long long tokens = (long long)dm.B * n;
    // short token rows: four tokens per wave (a flushed buffer has too few tokens to fill the chip that way)
    if (dm.H <= 8 && !dm.vhead && tokens >= GEAR_ROWS_MIN_TOKENS) {
      const int tpw = tokens >= (1 << 18) ? 4 : tokens >= (1 << 16) ? 2 : 1;   // >= 4096 blocks before a block takes more tokens
      // (the (scale, zero) array exists only under the per-vector grouping)
      hipLaunchKernelGGL(v_select_rows_kernel, dim3((n + 16 * tpw - 1) / (16 * tpw), dm.B), dim3(256), 0, st, V, dm.H, n, tpw,
                         kt, kb, thrV, dm.kcvt ? vsz : (uint32_t*)nullptr, dm.qmax);
      e = hipGetLastError();
    } else if (nc <= 2) e = launch_vsel<2>(V, dm, n, kt, kb, thrV, vsz, st);
    else if (nc <= 4) e = launch_vsel<4>(V, dm, n, kt, kb, thrV, vsz, st);
    else if (nc <= 8) e = launch_vsel<8>(V, dm, n, kt, kb, thrV, vsz, st);
    else if (nc <= 10) e = launch_vsel<10>(V, dm, n, kt, kb, thrV, vsz, st);
    else e = launch_vsel<16>(V, dm, n, kt, kb, thrV, vsz, st);
    if (e != hipSuccess) return e;
  }
  dim3 grid((n + TILE - 1) / TILE, dm.B * dm.H);
  if (dm.bits == 2)
    hipLaunchKernelGGL(v_quant_kernel<2>, grid, dim3(256), 0, st, V, sv, dm, n, (const ThreshPair*)thrV, (const uint32_t*)vsz,
                       k_top, k_bot, pool_ctr, Yout);
  else
    hipLaunchKernelGGL(v_quant_kernel<4>, grid, dim3(256), 0, st, V, sv, dm, n, (const ThreshPair*)thrV, (const uint32_t*)vsz,
                       k_top, k_bot, pool_ctr, Yout);
  return hipGetLastError();
}

}  // namespace gear
