// gear_decompress (X-hat = D + A B^T + S, Algorithm 1) and the canonical export
// views of the stored components.
#include "gear_internal.h"
#include "gear_launch.h"

namespace gear {

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

hipError_t launch_fill_u32(uint32_t* p, uint32_t v, size_t count, hipStream_t st) {
  if (count == 0) return hipSuccess;
  size_t blocks = (count + 255) / 256;
  if (blocks > 65535) blocks = 65535;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, v, count);
  return hipGetLastError();
}

__device__ __forceinline__ uint32_t load_code(const SegView& sv, const Dims& dm, bool is_k, int slab, int t,
                                              int c) {
  const uint32_t cmask = (1u << dm.bits) - 1u;
  if (is_k) {
    const int per = 32 / dm.bits;
    const uint32_t w = sv.codes[((size_t)slab * sv.n_cap + t) * dm.wpr + c / per];
    return (w >> ((c % per) * dm.bits)) & cmask;
  }
  const int tgg = t / dm.tpw, i = t - tgg * dm.tpw;
  const uint32_t w =
      sv.codes[((size_t)slab * sv.nblk_cap + (tgg >> 2)) * 512 + ((tgg & 3) * 16 + (c & 15)) * 8 + (c >> 4)];
  return (w >> (i * dm.bits)) & cmask;
}
__device__ __forceinline__ uint32_t load_sz(const SegView& sv, const Dims& dm, bool is_k, int slab, int t, int c) {
  if (is_k) return sv.sz[((size_t)slab * sv.ng_cap + key_group(dm, t)) * D + c];
  return sv.sz[((size_t)slab * sv.n_cap + t) * (D / dm.g) + c / dm.g];
}

// Calls f(row in the tile, channel, fp16 bits) for every filled fixed slot of one
// 64-token tile; the slots are spread over the 256 threads of the block.
template <class F>
__device__ __forceinline__ void for_each_ell(const SegView& sv, int is_k, int slab, int tile, int tid, F&& f) {
  if (is_k) {
    for (int i = tid; i < TILE * ELL_K; i += 256) {
      const int tl = i / ELL_K, t = tile * TILE + tl;
      if (t >= sv.n) continue;
      const uint32_t en = sv.ell[((size_t)slab * sv.n_cap + t) * ELL_K + (i % ELL_K)];
      if (en & ELL_VALID) f(tl, (int)(en & 127u), en >> 16);
    }
  } else {
    for (int i = tid; i < D * ELL_V; i += 256) {
      const int c = i / ELL_V;
      const uint32_t en = sv.ell[(((size_t)slab * sv.ntile_cap + tile) * D + c) * ELL_V + (i % ELL_V)];
      if ((en & ELL_VALID) && tile * TILE + (int)(en & 63u) < sv.n) f((int)(en & 63u), c, en >> 16);
    }
  }
}

// grid (ceil(n/64), B*H), block 256.
__global__ __launch_bounds__(256) void decompress_kernel(Dims dm, SegView sv, int is_k, uint16_t* __restrict__ out,
                                                         int n_total) {
  __shared__ float sp[TILE][D];
  __shared__ float Bs[D][8];
  const int slab = blockIdx.y, tile = blockIdx.x;
  const int b = slab / dm.H;
  const int tid = threadIdx.x;
  for (int i = tid; i < TILE * D; i += 256) sp[i / D][i % D] = 0.0f;
  for (int i = tid; i < D * 8; i += 256) {
    const int c = i >> 3, r = i & 7;
    Bs[c][r] = r < sv.rank ? h2f(sv.Bf[((size_t)slab * D + c) * sv.rank + r]) : 0.0f;
  }
  block_lds_sync();
  if (dm.ppm > 0) {
    const uint2 oc = sv.sp_table[(size_t)slab * sv.ntile_cap + tile];
    const uint32_t* lst = sv.sp_pool + (size_t)(is_k ? slab : b) * sv.pool_cap + oc.x;
    for (uint32_t e = tid; e < oc.y; e += 256) {
      const uint32_t en = lst[e];
      sp[(en & 0xFFFFu) >> 7][en & 127u] = h2f(en >> 16);
    }
    for_each_ell(sv, is_k, slab, tile, tid, [&](int tl, int c, uint32_t hb) { sp[tl][c] = h2f(hb); });
  }
  block_lds_sync();
  for (int i = tid; i < TILE * D; i += 256) {
    const int tl = i / D, c = i % D, t = tile * TILE + tl;
    if (t >= sv.n) break;
    const uint32_t sb = load_sz(sv, dm, is_k, slab, t, c);
    float v = (float)load_code(sv, dm, is_k, slab, t, c) * h2f(sb & 0xFFFFu) + h2f(sb >> 16);
    float lr = 0.0f;
    for (int r = 0; r < sv.rank; ++r) lr += h2f(sv.A[((size_t)slab * sv.n_cap + t) * sv.rank + r]) * Bs[c][r];
    v = v + lr + sp[tl][c];
    out[((size_t)slab * n_total + sv.t0 + t) * D + c] = (uint16_t)f2h(v);
  }
}

// grid (ceil(n/64), B*H), block 256.
__global__ __launch_bounds__(256) void export_codes_kernel(Dims dm, SegView sv, int is_k, uint8_t* __restrict__ codes,
                                                           uint16_t* __restrict__ scale, uint16_t* __restrict__ zero,
                                                           int n_total, int ng_total) {
  const int slab = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  for (int i = tid; i < TILE * D; i += 256) {
    const int tl = i / D, c = i % D, t = tile * TILE + tl;
    if (t >= sv.n) break;
    codes[((size_t)slab * n_total + sv.t0 + t) * D + c] = (uint8_t)load_code(sv, dm, is_k, slab, t, c);
    const uint32_t sb = load_sz(sv, dm, is_k, slab, t, c);
    if (is_k) {
      if (dm.kcvt ? t == 0 : t % dm.g == 0) {
        const size_t o = ((size_t)slab * ng_total + sv.g0 + key_group(dm, t)) * D + c;
        scale[o] = (uint16_t)(sb & 0xFFFFu);
        zero[o] = (uint16_t)(sb >> 16);
      }
    } else if (c % dm.g == 0) {
      const size_t o = ((size_t)slab * n_total + sv.t0 + t) * (D / dm.g) + c / dm.g;
      scale[o] = (uint16_t)(sb & 0xFFFFu);
      zero[o] = (uint16_t)(sb >> 16);
    }
  }
}

// grid (ceil(n/64), B*H), block 256.  Outputs must be zero-filled beforehand.
__global__ __launch_bounds__(256) void export_sparse_kernel(Dims dm, SegView sv, int is_k, uint8_t* __restrict__ mask,
                                                            uint16_t* __restrict__ vals, int n_total) {
  const int slab = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  const int b = slab / dm.H;
  const uint2 oc = sv.sp_table[(size_t)slab * sv.ntile_cap + tile];
  const uint32_t* lst = sv.sp_pool + (size_t)(is_k ? slab : b) * sv.pool_cap + oc.x;
  for (uint32_t e = tid; e < oc.y; e += 256) {
    const uint32_t en = lst[e];
    const int t = tile * TILE + (int)((en & 0xFFFFu) >> 7), c = en & 127u;
    if (t < sv.n) {
      const size_t o = ((size_t)slab * n_total + sv.t0 + t) * D + c;
      mask[o] = 1;
      vals[o] = (uint16_t)(en >> 16);
    }
  }
  for_each_ell(sv, is_k, slab, tile, tid, [&](int tl, int c, uint32_t hb) {
    const size_t o = ((size_t)slab * n_total + sv.t0 + tile * TILE + tl) * D + c;
    mask[o] = 1;
    vals[o] = (uint16_t)hb;
  });
}

// ---- COO view of S: (linear index into [B, H, n_total, 128], fp16 value), sorted by index ----
// Pass 1 (count = 1) leaves the number of outliers of every token row in rowcnt[slab * n_total + t];
// after the prefix sums, pass 2 (count = 0) writes each row's entries in channel order from rowcnt[row]
// (then the row's first position).  grid (ceil(n/64), B*H), block 256: the tile's part of S is
// rebuilt in LDS as a bit per entry plus its value.
__global__ __launch_bounds__(256) void coo_tile_kernel(Dims dm, SegView sv, int is_k, int count, uint32_t* __restrict__ rowcnt,
                                                       long long* __restrict__ lin, uint16_t* __restrict__ vals, int n_total) {
  __shared__ uint32_t bits[TILE][4];
  __shared__ uint16_t val[TILE][D];
  const int slab = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
  const int b = slab / dm.H;
  if (tid < TILE * 4) (&bits[0][0])[tid] = 0u;
  block_lds_sync();
  auto put = [&](int tl, int c, uint32_t hb) {
    atomicOr(&bits[tl][c >> 5], 1u << (c & 31));
    val[tl][c] = (uint16_t)hb;
  };
  if (dm.ppm > 0) {
    const uint2 oc = sv.sp_table[(size_t)slab * sv.ntile_cap + tile];
    const uint32_t* lst = sv.sp_pool + (size_t)(is_k ? slab : b) * sv.pool_cap + oc.x;
    for (uint32_t e = tid; e < oc.y; e += 256) {
      const uint32_t en = lst[e];
      const int tl = (int)((en & 0xFFFFu) >> 7);
      if (tile * TILE + tl < sv.n) put(tl, (int)(en & 127u), en >> 16);
    }
    for_each_ell(sv, is_k, slab, tile, tid, put);
  }
  block_lds_sync();
  if (tid < TILE && tile * TILE + tid < sv.n) {
    const size_t row = (size_t)slab * n_total + sv.t0 + tile * TILE + tid;
    if (count) {
      rowcnt[row] = __popc(bits[tid][0]) + __popc(bits[tid][1]) + __popc(bits[tid][2]) + __popc(bits[tid][3]);
    } else {
      size_t o = rowcnt[row];
      for (int w = 0; w < 4; ++w) {
        uint32_t m = bits[tid][w];
        while (m) {
          const int c = 32 * w + __ffs((int)m) - 1;
          m &= m - 1u;
          lin[o] = (long long)(row * D + c);
          vals[o] = val[tid][c];
          ++o;
        }
      }
    }
  }
}

// Exclusive prefix sums of v[0 .. count) in place, in three launches: sums of chunks of 1024,
// their prefix sums (one block), then each chunk's own scan.
__global__ __launch_bounds__(256) void scan_chunk_sums_kernel(const uint32_t* __restrict__ v, size_t count, uint32_t* __restrict__ sums) {
  __shared__ uint32_t red[4];
  const size_t base = (size_t)blockIdx.x * 1024;
  uint32_t s = 0;
  for (int i = threadIdx.x; i < 1024; i += 256)
    if (base + i < count) s += v[base + i];
  s = wave_sum_shfl(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  block_lds_sync();
  if (threadIdx.x == 0) sums[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
__global__ __launch_bounds__(256) void scan_sums_kernel(uint32_t* __restrict__ sums, int nchunks) {   // one block
  __shared__ uint32_t wtot[4];
  __shared__ uint32_t carry_s;
  if (threadIdx.x == 0) carry_s = 0u;
  block_lds_sync();
  for (int i0 = 0; i0 < nchunks; i0 += 256) {
    const int i = i0 + threadIdx.x;
    const uint32_t x = i < nchunks ? sums[i] : 0u;
    const uint32_t inc = wave_incl_scan(x);
    if ((threadIdx.x & 63) == 63) wtot[threadIdx.x >> 6] = inc;
    block_lds_sync();
    uint32_t off = carry_s;
    for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) off += wtot[w];
    if (i < nchunks) sums[i] = off + inc - x;
    block_lds_sync();
    if (threadIdx.x == 255) carry_s = off + inc;
    block_lds_sync();
  }
}
__global__ __launch_bounds__(256) void scan_apply_kernel(uint32_t* __restrict__ v, size_t count, const uint32_t* __restrict__ sums) {
  __shared__ uint32_t wtot[4];
  const size_t base = (size_t)blockIdx.x * 1024 + (size_t)threadIdx.x * 4;
  uint32_t x[4], t = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[i] = base + i < count ? v[base + i] : 0u;
    t += x[i];
  }
  const uint32_t inc = wave_incl_scan(t);
  if ((threadIdx.x & 63) == 63) wtot[threadIdx.x >> 6] = inc;
  block_lds_sync();
  uint32_t off = sums[blockIdx.x] + inc - t;
  for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) off += wtot[w];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (base + i < count) v[base + i] = off;
    off += x[i];
  }
}

__global__ void export_lowrank_kernel(SegView sv, uint16_t* __restrict__ A, uint16_t* __restrict__ Bf, int slabs) {
  const size_t na = (size_t)slabs * sv.n * sv.rank, nb = (size_t)slabs * D * sv.rank;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < na + nb; i += (size_t)gridDim.x * blockDim.x) {
    if (i < na) {
      const size_t per = (size_t)sv.n * sv.rank;
      const size_t slab = i / per, r = i - slab * per;
      A[i] = sv.A[slab * sv.n_cap * sv.rank + r];
    } else {
      Bf[i - na] = sv.Bf[i - na];
    }
  }
}

hipError_t launch_decompress(const Dims& dm, const SegView& ks, const SegView& vs, uint16_t* Kout,
                             uint16_t* Vout, int n_total, hipStream_t st) {
  dim3 grid((ks.n + TILE - 1) / TILE, dm.B * dm.H);
  if (Kout) hipLaunchKernelGGL(decompress_kernel, grid, dim3(256), 0, st, dm, ks, 1, Kout, n_total);
  if (Vout) hipLaunchKernelGGL(decompress_kernel, grid, dim3(256), 0, st, dm, vs, 0, Vout, n_total);
  return hipGetLastError();
}

hipError_t launch_export_codes(const Dims& dm, const SegView& sv, bool is_k, uint8_t* codes, uint16_t* scale,
                               uint16_t* zero, int n_total, int ng_total, hipStream_t st) {
  dim3 grid((sv.n + TILE - 1) / TILE, dm.B * dm.H);
  hipLaunchKernelGGL(export_codes_kernel, grid, dim3(256), 0, st, dm, sv, is_k ? 1 : 0, codes, scale, zero,
                     n_total, ng_total);
  return hipGetLastError();
}

hipError_t launch_export_sparse(const Dims& dm, const SegView& sv, bool is_k, uint8_t* mask, uint16_t* vals,
                                int n_total, hipStream_t st) {
  if (dm.ppm == 0) return hipSuccess;
  dim3 grid((sv.n + TILE - 1) / TILE, dm.B * dm.H);
  hipLaunchKernelGGL(export_sparse_kernel, grid, dim3(256), 0, st, dm, sv, is_k ? 1 : 0, mask, vals, n_total);
  return hipGetLastError();
}

hipError_t launch_coo_tiles(const Dims& dm, const SegView& sv, bool is_k, bool count, uint32_t* rowcnt, long long* lin,
                            uint16_t* vals, int n_total, hipStream_t st) {
  dim3 grid((sv.n + TILE - 1) / TILE, dm.B * dm.H);
  hipLaunchKernelGGL(coo_tile_kernel, grid, dim3(256), 0, st, dm, sv, is_k ? 1 : 0, count ? 1 : 0, rowcnt, lin, vals, n_total);
  return hipGetLastError();
}

hipError_t launch_exclusive_scan(uint32_t* v, size_t count, uint32_t* sums, hipStream_t st) {
  const int nchunks = (int)((count + 1023) / 1024);
  if (nchunks == 0) return hipSuccess;
  hipLaunchKernelGGL(scan_chunk_sums_kernel, dim3(nchunks), dim3(256), 0, st, (const uint32_t*)v, count, sums);
  hipLaunchKernelGGL(scan_sums_kernel, dim3(1), dim3(256), 0, st, sums, nchunks);
  hipLaunchKernelGGL(scan_apply_kernel, dim3(nchunks), dim3(256), 0, st, v, count, (const uint32_t*)sums);
  return hipGetLastError();
}

hipError_t launch_export_lowrank(const Dims& dm, const SegView& sv, uint16_t* A, uint16_t* Bf, hipStream_t st) {
  if (sv.rank == 0) return hipSuccess;
  hipLaunchKernelGGL(export_lowrank_kernel, dim3(1024), dim3(256), 0, st, sv, A, Bf, dm.B * dm.H);
  return hipGetLastError();
}

}  // namespace gear
