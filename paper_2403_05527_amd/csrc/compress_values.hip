// Filter_s (Eq. 4) + Quant_b(X - S) (Eq. 2 / Eq. 5) kernels of gear_compress, Value side:
//   v_select_kernel  thresholds of every Value token vector: the token's row over
//                    ALL heads' channels (index j = h*128 + c), one wave per token
//                    with the vector in registers
//   v_quant_kernel   per (b, h, 64-token tile): outlier predicate, per-token group
//                    min/max inside the row (lane exchanges), codes written in the
//                    token-blocked order the decode kernel's MFMA operand expects,
//                    (scale, zero), the tile's outlier list ordered (c, t), residual
#include "gear_internal.h"
#include "gear_select.h"
#include "gear_launch.h"

namespace gear {

template <int NC>
struct RegSource {  // the vector lives in the wave's registers
  static constexpr int kMaxChunks = NC;
  const uint4* x;
  __device__ __forceinline__ uint4 operator()(int ch) const { return x[ch]; }
};

constexpr int VSEL_TOKENS = 16;  // tokens per block (4 per wave)

// grid (ceil(n/16), B); block 256.  lane l, chunk ch  <->  head 4*ch + l/16,
// channels 8*(l%16)..+7, i.e. in-vector index ch*512 + l*8 + e.
template <int NC>
__global__ __launch_bounds__(256) void v_select_kernel(const uint16_t* __restrict__ V, int H, int n, int k_top,
                                                       int k_bot, Thresh* __restrict__ thrV) {
  __shared__ uint32_t hist[4 * 512];
  const int b = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hsub = lane >> 4, oc = lane & 15;
  const int N = H * D;
  for (int i = 0; i < VSEL_TOKENS / 4; ++i) {
    const int t = blockIdx.x * VSEL_TOKENS + i * 4 + wave;
    const bool tvalid = t < n;
    uint4 x[NC];
#pragma unroll
    for (int ch = 0; ch < NC; ++ch) {
      const int head = 4 * ch + hsub;
      x[ch] = make_uint4(0, 0, 0, 0);
      if (tvalid && head < H) {
        const uint4 raw = *reinterpret_cast<const uint4*>(V + (((size_t)(b * H + head) * n + t) * D + oc * 8));
        x[ch] = make_uint4(key16x2(raw.x), key16x2(raw.y), key16x2(raw.z), key16x2(raw.w));
      }
    }
    RegSource<NC> src{x};
    const Thresh th = wave_select(src, N, k_top, k_bot, hist + wave * 512, tvalid);
    if (tvalid && lane == 0) thrV[(size_t)b * n + t] = th;
  }
}

// grid (ceil(n/64), B*H); block 256; thread (r0 = tid/16, oc = tid%16) owns
// channels 8*oc..+7 of rows t0 + r0 + 16*k, k = 0..3.
__global__ __launch_bounds__(256) void v_quant_kernel(const uint16_t* __restrict__ V, SegView sv, Dims dm, int n,
                                                      const Thresh* __restrict__ thrV, uint32_t* __restrict__ pool_ctr,
                                                      uint16_t* __restrict__ Rout, uint8_t* __restrict__ Rlo) {
  constexpr int PITCH = 136;  // bytes per staged code row (multiple of 8)
  __shared__ __align__(16) uint8_t stage[TILE * PITCH];
  __shared__ uint32_t colmask[D][2];
  __shared__ uint32_t wtot[2];
  __shared__ uint32_t list_off;
  const int slab = blockIdx.y, tile = blockIdx.x;
  const int b = slab / dm.H, h = slab - b * dm.H;
  const int t0 = tile * TILE;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const int g = dm.g, bits = dm.bits, tpw = dm.tpw;
  const uint16_t* X = V + (size_t)slab * n * D;

  if (tid < D) { colmask[tid][0] = 0u; colmask[tid][1] = 0u; }
  block_lds_sync();

  // every row of the tile and its thresholds are requested before the first one is used
  uint4 xrow[4];
  Thresh trow[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int t = t0 + r0 + 16 * k;
    xrow[k] = make_uint4(0, 0, 0, 0);
    trow[k] = thresh_none();
    if (t < n) {
      xrow[k] = *reinterpret_cast<const uint4*>(X + (size_t)t * D + oc * 8);
      if (dm.ppm > 0) trow[k] = thrV[(size_t)b * n + t];
    }
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int tl = r0 + 16 * k, t = t0 + tl;
    const bool tv = t < n;
    const uint4 xv = xrow[k];
    const ThreshPair th = pack_thresh(trow[k]);
    const uint32_t w[4] = {xv.x, xv.y, xv.z, xv.w};
    float y[8];
    float lmn = INFINITY, lmx = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t hb = (w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
      const int c = oc * 8 + e;
      const bool out = tv && is_outlier(key16(hb), (uint32_t)(h * D + c), th);
      if (out) atomicOr(&colmask[c][tl >> 5], 1u << (tl & 31));
      y[e] = out ? 0.0f : h2f(hb);
      lmn = fminf(lmn, y[e]);
      lmx = fmaxf(lmx, y[e]);
    }
    // group = g consecutive channels of the row = g/8 neighbouring lanes
    lmn = fminf(lmn, dpp_f<DPP_XOR1>(lmn));
    lmx = fmaxf(lmx, dpp_f<DPP_XOR1>(lmx));
    lmn = fminf(lmn, dpp_f<DPP_XOR2>(lmn));
    lmx = fmaxf(lmx, dpp_f<DPP_XOR2>(lmx));
    if (g >= 64) {
      lmn = fminf(lmn, dpp_f<DPP_HALF_MIRROR>(lmn));
      lmx = fmaxf(lmx, dpp_f<DPP_HALF_MIRROR>(lmx));
    }
    if (g >= 128) {
      lmn = fminf(lmn, dpp_f<DPP_MIRROR>(lmn));
      lmx = fmaxf(lmx, dpp_f<DPP_MIRROR>(lmx));
    }
    const GroupQ q = make_group(lmn, lmx, dm.qmax);
    uint32_t cb[2] = {0u, 0u};   // 8 code bytes
    uint32_t rh[8], rl[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t code = quant_code_resid(y[e], q, dm.qmax, rh[e], rl[e]);
      cb[e >> 2] |= (tv ? code : 0u) << ((e & 3) * 8);
    }
    *reinterpret_cast<uint2*>(&stage[tl * PITCH + oc * 8]) = make_uint2(cb[0], cb[1]);
    if (tv) {
      if ((oc & ((g >> 3) - 1)) == 0) sv.sz[((size_t)slab * sv.n_cap + t) * (D / g) + (oc * 8) / g] = group_bits(q);
      if (Rout) {
        const size_t ro = ((size_t)slab * n + t) * D + oc * 8;
        *reinterpret_cast<uint4*>(Rout + ro) =
            make_uint4(rh[0] | (rh[1] << 16), rh[2] | (rh[3] << 16), rh[4] | (rh[5] << 16), rh[6] | (rh[7] << 16));
        *reinterpret_cast<uint2*>(Rlo + ro) = make_uint2(rl[0] | (rl[1] << 8) | (rl[2] << 16) | (rl[3] << 24),
                                                         rl[4] | (rl[5] << 8) | (rl[6] << 16) | (rl[7] << 24));
      }
    }
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
      const uint32_t off = atomicAdd(&pool_ctr[b], tot);
      sv.sp_table[(size_t)slab * sv.ntile_cap + tile] = make_uint2(off, tot);
      list_off = off;
    }
    block_lds_sync();
    if (tid < D) {
      uint32_t off = list_off + (wave == 1 ? wtot[0] : 0u) + inc - cnt;
      uint32_t* pool = sv.sp_pool + (size_t)b * sv.pool_cap;
      uint32_t* slots = sv.ell + (((size_t)slab * sv.ntile_cap + tile) * D + tid) * ELL_V;
      uint32_t s_i = 0;
      for (int half = 0; half < 2; ++half) {
        uint32_t mm = half ? m1 : m0;
        while (mm) {
          const int bit = __ffs((int)mm) - 1;
          mm &= mm - 1;
          const int tl = half * 32 + bit;
          const uint32_t hb = X[(size_t)(t0 + tl) * D + tid];
          if (s_i < ELL_V) {
            slots[s_i] = (uint32_t)tl | ELL_VALID | (hb << 16);
          } else {
            if (off < sv.pool_cap) pool[off] = (uint32_t)(tl * D + tid) | (hb << 16);
            ++off;
          }
          ++s_i;
        }
      }
      for (; s_i < ELL_V; ++s_i) slots[s_i] = 0u;   // empty slots
    }
  }
}

// ------------------------------------------------------------------ launchers
template <int NC>
static hipError_t launch_vsel(const uint16_t* V, const Dims& dm, int n, int k_top, int k_bot, Thresh* thrV,
                              hipStream_t st) {
  dim3 grid((n + VSEL_TOKENS - 1) / VSEL_TOKENS, dm.B);
  hipLaunchKernelGGL(v_select_kernel<NC>, grid, dim3(256), 0, st, V, dm.H, n, k_top, k_bot, thrV);
  return hipGetLastError();
}

hipError_t launch_v_filter_quant(const uint16_t* V, const SegView& sv, const Dims& dm, int n, int k_top,
                                 int k_bot, Thresh* thrV, uint32_t* pool_ctr, uint16_t* Rout, uint8_t* Rlo,
                                 hipStream_t st) {
  if (dm.ppm > 0) {
    const int nc = (dm.H + 3) / 4;
    hipError_t e;
    if (nc <= 2) e = launch_vsel<2>(V, dm, n, k_top, k_bot, thrV, st);
    else if (nc <= 4) e = launch_vsel<4>(V, dm, n, k_top, k_bot, thrV, st);
    else if (nc <= 8) e = launch_vsel<8>(V, dm, n, k_top, k_bot, thrV, st);
    else if (nc <= 10) e = launch_vsel<10>(V, dm, n, k_top, k_bot, thrV, st);
    else e = launch_vsel<16>(V, dm, n, k_top, k_bot, thrV, st);
    if (e != hipSuccess) return e;
  }
  dim3 grid((n + TILE - 1) / TILE, dm.B * dm.H);
  hipLaunchKernelGGL(v_quant_kernel, grid, dim3(256), 0, st, V, sv, dm, n, (const Thresh*)thrV, pool_ctr, Rout, Rlo);
  return hipGetLastError();
}

}  // namespace gear
