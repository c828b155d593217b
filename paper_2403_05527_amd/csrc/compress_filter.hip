// Filter_s (Eq. 4) + Quant_b(X - S) (Eq. 2 / Eq. 5) kernels of gear_compress, Key side:
//   k_select_kernel       thresholds of every Key channel vector (over tokens)
//   k_quant_kernel        Key codes, (scale, zero), ordered outlier lists, residual
// (the Value side is in compress_values.hip)
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
// 1-D grid of (128/CB) * B*H blocks of 64 * min(CB, 4) threads; LDS: 512 u32 per wave + [CB][n_pad] keys.
// Consecutive block ids go round-robin to the chip's 8 XCDs (each with its own L2), so
// the id is decoded with the column block fastest INSIDE one XCD: the 128/CB blocks
// that share the 128-byte lines of one slab then meet in one L2 instead of eight.
__global__ __launch_bounds__(256) void k_select_kernel(const uint16_t* __restrict__ K, int n, int n_pad,
                                                       int CB, int nslab, int k_top, int k_bot,
                                                       Thresh* __restrict__ thrK) {
  GEAR_DYN_LDS(smem_raw);
  uint32_t* hist_all = reinterpret_cast<uint32_t*>(smem_raw);
  uint16_t* tile = reinterpret_cast<uint16_t*>(smem_raw + (blockDim.x >> 6) * 512 * sizeof(uint32_t));
  const int ncb = D / CB;
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

  // transpose-load the [n x CB] column block so every vector is contiguous; a
  // thread has UNR row segments in flight at a time
  const int VW = CB < 8 ? CB : 8;   // fp16 values per row segment
  const int U = CB / VW;
  {
    constexpr int UNR = 8;
    const int total = n * U;
    for (int base = 0; base < total; base += NT * UNR) {
      uint4 q[UNR];
#pragma unroll
      for (int k = 0; k < UNR; ++k) {
        const int idx = base + k * NT + tid;
        q[k] = make_uint4(0, 0, 0, 0);
        if (idx < total) {
          const int row = idx / U, u = idx - row * U;
          const uint16_t* p = X + (size_t)row * D + u * VW;
          if (VW == 8) {
            q[k] = *reinterpret_cast<const uint4*>(p);
          } else if (VW == 4) {
            const uint2 t2 = *reinterpret_cast<const uint2*>(p);
            q[k].x = t2.x; q[k].y = t2.y;
          } else if (VW == 2) {
            q[k].x = *reinterpret_cast<const uint32_t*>(p);
          } else {
            q[k].x = *p;
          }
        }
      }
#pragma unroll
      for (int k = 0; k < UNR; ++k) {
        const int idx = base + k * NT + tid;
        if (idx < total) {
          const int row = idx / U, u = idx - row * U;
          const uint32_t w[4] = {key16x2(q[k].x), key16x2(q[k].y), key16x2(q[k].z), key16x2(q[k].w)};
          uint16_t* dst = tile + (size_t)(u * VW) * n_pad + row;
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (e < VW) dst[(size_t)e * n_pad] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));   // keys, not values
        }
      }
    }
  }
  // zero the padding so stray lanes read defined data
  for (int idx = tid; idx < CB * (n_pad - n); idx += NT) {
    const int c = idx / (n_pad - n), r = idx - c * (n_pad - n);
    tile[(size_t)c * n_pad + n + r] = 0;
  }
  block_lds_sync();

  const int iters = (CB + NW - 1) / NW;
  for (int it = 0; it < iters; ++it) {
    const int v = it * NW + wave;
    const bool active = v < CB;
    LdsSource src{tile + (size_t)(active ? v : 0) * n_pad, n_pad};
    const Thresh th = wave_select(src, n, k_top, k_bot, hist_all + wave * 512, active);
    if (active && lane == 0) thrK[(size_t)slab * D + cb * CB + v] = th;
  }
}

// ------------------------------------------------------------------ K quant
// Entry e of a row piece after the Filter: X - S, i.e. 0 where the entry is an outlier
// (re-derived from the raw words where needed instead of being kept in registers).
__device__ __forceinline__ float yval(const uint32_t* raw4, uint32_t flags, int e) {
  const uint32_t hb = (raw4[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
  return (flags & (1u << e)) ? 0.0f : h2f(hb);
}
// grid (ceil(n/WT), B*H); block 256; WT = max(64, g) tokens per block.
// thread (r0 = tid/16, oc = tid%16) owns channels 8*oc..8*oc+7 of rows
// t0 + r0 + 16*k.
template <int WT>
__global__ __launch_bounds__(256, (WT == 64 ? 3 : 2)) void k_quant_kernel(const uint16_t* __restrict__ K, SegView sv, Dims dm,
                                                      int n, const Thresh* __restrict__ thrK,
                                                      uint32_t* __restrict__ pool_ctr,
                                                      uint16_t* __restrict__ Rout, uint8_t* __restrict__ Rlo) {
  constexpr int NK = WT / 16;
  __shared__ float red_mn[4][D];
  __shared__ float red_mx[4][D];
  __shared__ float gq_mn[2][D];
  __shared__ float gq_inv[2][D];
  __shared__ uint32_t band_cnt[NK][4];
  __shared__ uint32_t tile_off[2];

  const int slab = blockIdx.y;
  const int t0 = blockIdx.x * WT;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const uint16_t* X = K + (size_t)slab * n * D;
  const int g = dm.g;
  const int ngw = WT / g;  // groups per block (1 or 2)

  // thresholds of my 8 channels (staged through LDS: one coalesced read per block)
  uint32_t raw[NK][4];
  uint32_t flags[NK];
  // every row of the tile is requested before the first one is used
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const int t = t0 + r0 + 16 * k;
    uint4 q = make_uint4(0, 0, 0, 0);
    if (t < n) q = *reinterpret_cast<const uint4*>(X + (size_t)t * D + oc * 8);
    raw[k][0] = q.x; raw[k][1] = q.y; raw[k][2] = q.z; raw[k][3] = q.w;
  }
  // thresholds of my 8 channels (staged through LDS: one coalesced read per block)
  __shared__ ThreshPair thr_s[D];
  if (tid < D) thr_s[tid] = pack_thresh(dm.ppm > 0 ? thrK[(size_t)slab * D + tid] : thresh_none());
  block_lds_sync();
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const int t = t0 + r0 + 16 * k;
    flags[k] = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t hb = (raw[k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
      const bool out = (t < n) && is_outlier(key16(hb), (uint32_t)t, thr_s[oc * 8 + e]);   // read per use: saves 16 registers
      if (out) flags[k] |= 1u << e;
    }
  }

  // group min / max per channel
  for (int gi = 0; gi < ngw; ++gi) {
    float lmn[8], lmx[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { lmn[e] = INFINITY; lmx[e] = -INFINITY; }
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int tl = r0 + 16 * k;
      if (tl / g == gi && t0 + tl < n) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float yv = yval(raw[k], flags[k], e);
          lmn[e] = fminf(lmn[e], yv);
          lmx[e] = fmaxf(lmx[e], yv);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      lmn[e] = fminf(lmn[e], __shfl_xor(lmn[e], 16, 64));
      lmn[e] = fminf(lmn[e], __shfl_xor(lmn[e], 32, 64));
      lmx[e] = fmaxf(lmx[e], __shfl_xor(lmx[e], 16, 64));
      lmx[e] = fmaxf(lmx[e], __shfl_xor(lmx[e], 32, 64));
    }
    if (lane < 16) {
#pragma unroll
      for (int e = 0; e < 8; ++e) { red_mn[wave][oc * 8 + e] = lmn[e]; red_mx[wave][oc * 8 + e] = lmx[e]; }
    }
    block_lds_sync();
    if (tid < D && t0 + gi * g < n) {
      const float mn = fminf(fminf(red_mn[0][tid], red_mn[1][tid]), fminf(red_mn[2][tid], red_mn[3][tid]));
      const float mx = fmaxf(fmaxf(red_mx[0][tid], red_mx[1][tid]), fmaxf(red_mx[2][tid], red_mx[3][tid]));
      const GroupQ q = make_group(mn, mx, dm.qmax);
      gq_mn[gi][tid] = q.mn;
      gq_inv[gi][tid] = q.inv;
      const int grp = (t0 + gi * g) / g;
      sv.sz[((size_t)slab * sv.ng_cap + grp) * D + tid] = group_bits(q);
    }
    block_lds_sync();
  }

  // codes, packed token-major
  uint32_t* crow = sv.codes + (size_t)slab * sv.n_cap * dm.wpr;
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const int tl = r0 + 16 * k, t = t0 + tl;
    if (t < n) {
      const int gi = tl / g;
      uint32_t w = 0;
      uint32_t rh[8], rl[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        GroupQ q;
        q.mn = gq_mn[gi][oc * 8 + e];
        q.inv = gq_inv[gi][oc * 8 + e];
        q.delta = 0.0f;
        const uint32_t code = quant_code_resid(yval(raw[k], flags[k], e), q, dm.qmax, rh[e], rl[e]);   // residual R = u * delta
        w |= code << (e * dm.bits);
      }
      if (Rout) {
        *reinterpret_cast<uint4*>(Rout + ((size_t)slab * n + t) * D + oc * 8) =
            make_uint4(rh[0] | (rh[1] << 16), rh[2] | (rh[3] << 16), rh[4] | (rh[5] << 16), rh[6] | (rh[7] << 16));
        *reinterpret_cast<uint2*>(Rlo + ((size_t)slab * n + t) * D + oc * 8) =
            make_uint2(rl[0] | (rl[1] << 8) | (rl[2] << 16) | (rl[3] << 24),
                       rl[4] | (rl[5] << 8) | (rl[6] << 16) | (rl[7] << 24));
      }
      if (dm.bits == 4) {
        crow[(size_t)t * dm.wpr + oc] = w;
      } else {  // 2 bits: 16 bits per thread
        reinterpret_cast<uint16_t*>(crow + (size_t)t * dm.wpr)[oc] = (uint16_t)w;
      }
    }
  }

  // Outliers of a token row: the first ELL_K in channel order take the row's fixed
  // slots, the rest go to the tile's overflow list, ordered (t, c).  The 16 lanes
  // that own a row are 16 consecutive lanes.
  if (dm.ppm > 0) {
    uint32_t cnt[NK], inc[NK], pre[NK];   // overflow entries of this lane, their scan over the wave; outliers of the row before this lane
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const int t = t0 + r0 + 16 * k;
      const uint32_t c_all = __popc(flags[k]);
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
        uint32_t s_i = pre[k];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if ((flags[k] & (1u << e)) && s_i < ELL_K) {
            const uint32_t hb = (raw[k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
            slots[s_i] = (uint32_t)(oc * 8 + e) | ELL_VALID | (hb << 16);
            ++s_i;
          }
        }
        if (oc < ELL_K && (uint32_t)oc >= row_total) slots[oc] = 0u;   // empty slots
      }
      inc[k] = wave_incl_scan(cnt[k]);
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
      const int tl = r0 + 16 * k;
      const int ti = k / 4;  // tile inside the block
      uint32_t off = tile_off[ti];
      for (int kk = ti * 4; kk < k; ++kk)
        for (int w = 0; w < 4; ++w) off += band_cnt[kk][w];
      for (int w = 0; w < wave; ++w) off += band_cnt[k][w];
      off += inc[k] - cnt[k];
      uint32_t s_i = pre[k];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (flags[k] & (1u << e)) {
          if (s_i >= ELL_K) {
            const uint32_t hb = (raw[k][e >> 1] >> ((e & 1) * 16)) & 0xFFFFu;
            if (off < sv.pool_cap) pool[off] = (uint32_t)((tl & 63) * D + oc * 8 + e) | (hb << 16);
            ++off;
          }
          ++s_i;
        }
      }
    }
  }
}

// ------------------------------------------------------------------ launchers
constexpr size_t KSEL_TILE_BYTES = 32768;   // LDS tile of one block: 4 blocks per CU; smaller tiles mean 4-byte row pieces, measured slower
static int k_select_cb(int n_pad) {
  int cb = 128;
  while (cb > 1 && (size_t)cb * n_pad * 2 > KSEL_TILE_BYTES) cb >>= 1;
  return cb;
}

hipError_t launch_k_select(const uint16_t* K, const Dims& dm, int n, int k_top, int k_bot, Thresh* thrK,
                           hipStream_t st) {
  const int n_pad = (n + 7) & ~7;
  const int cb = k_select_cb(n_pad);
  const int nw = cb < 4 ? cb : 4;   // waves per block: one vector each per round
  const size_t lds = (size_t)nw * 512 * sizeof(uint32_t) + (size_t)cb * n_pad * 2;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_select_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  dim3 grid((D / cb) * dm.B * dm.H);
  hipLaunchKernelGGL(k_select_kernel, grid, dim3(64 * nw), lds, st, K, n, n_pad, cb, dm.B * dm.H, k_top, k_bot, thrK);
  return hipGetLastError();
}

hipError_t launch_k_quant(const uint16_t* K, const SegView& sv, const Dims& dm, int n, const Thresh* thrK,
                          uint32_t* pool_ctr, uint16_t* Rout, uint8_t* Rlo, hipStream_t st) {
  if (dm.g == 128) {
    dim3 grid((n + 127) / 128, dm.B * dm.H);
    hipLaunchKernelGGL(k_quant_kernel<128>, grid, dim3(256), 0, st, K, sv, dm, n, thrK, pool_ctr, Rout, Rlo);
  } else {
    dim3 grid((n + 63) / 64, dm.B * dm.H);
    hipLaunchKernelGGL(k_quant_kernel<64>, grid, dim3(256), 0, st, K, sv, dm, n, thrK, pool_ctr, Rout, Rlo);
  }
  return hipGetLastError();
}

}  // namespace gear
