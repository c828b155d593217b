// gear_decode_attn: single-query attention (Eq. 1) read directly from the
// compressed cache.  K-hat and V-hat are never materialised:
//   score_t = q . D_K[t] + (q^T B_K) . A_K[t] + q . S_K[t]
//   out     = sum_t p_t D_V[t] + (p^T A_V) B_V^T + p^T S_V
// (the low-rank term as a down- then up-projection, as the paper's
// implementation notes describe), followed by the fp16 buffer rows.
//
// Split-KV: block (split, b*H_kv + h) handles DECODE_SPLIT tokens of the prefill
// segment for all query heads of the KV head on the matrix cores
// (decode_mfma.h); the last split index handles the appended chunk segments and
// the fp16 buffer (decode_tail.h).  Every block writes one partial softmax
// record (m, l, o) per query head; decode_combine merges the records.
#include "gear_internal.h"
#include "gear_launch.h"
#include "decode_mfma.h"
#include "decode_tail.h"

namespace gear {

static_assert(MFMA_TS == DECODE_SPLIT, "split size is part of the workspace layout");

// grid (nsplit + 1, B*H_kv), block 256.
template <int BITS, int GQ>
__global__ __launch_bounds__(256, 4) void decode_split_kernel(Dims dm, SegView k0, SegView v0, ChunkSet cs,
                                                              const uint16_t* __restrict__ q,
                                                              const uint16_t* __restrict__ Kbuf,
                                                              const uint16_t* __restrict__ Vbuf, int n_buf,
                                                              int n_buf_cap, float* __restrict__ partial) {
  GEAR_DYN_LDS(smem_raw);
  const int slab = blockIdx.y, split = blockIdx.x;
  const int nsplit = (int)gridDim.x - 1;
  const int b = slab / dm.H, h = slab - b * dm.H;
  float* rec_base = partial + (((size_t)b * dm.Hq + h * GQ) * (nsplit + 1) + split) * DECODE_REC;
  const int rec_stride = (nsplit + 1) * DECODE_REC;
  const uint16_t* qg = q + ((size_t)b * dm.Hq + h * GQ) * D;
  if (split == nsplit) {
    tail_block<GQ>(*reinterpret_cast<TailSmem<GQ>*>(smem_raw), dm, cs, qg, Kbuf + (size_t)slab * n_buf_cap * D,
                   Vbuf + (size_t)slab * n_buf_cap * D, n_buf, slab, b, rec_base, rec_stride);
    return;
  }
  const int t_begin = split * MFMA_TS;
  const int t_end = min(k0.n, t_begin + MFMA_TS);
  mfma_block<BITS, GQ>(smem_raw, dm, k0, v0, qg, slab, b, t_begin, t_end, rec_base, rec_stride);
}

// grid (B*H_q), block 128.
__global__ __launch_bounds__(128) void decode_combine_kernel(const float* __restrict__ partial, int nrec,
                                                             uint16_t* __restrict__ out) {
  const int row = blockIdx.x, c = threadIdx.x;
  const float* rec = partial + (size_t)row * nrec * DECODE_REC;
  float M = -INFINITY;
  for (int s = 0; s < nrec; ++s) M = fmaxf(M, rec[(size_t)s * DECODE_REC]);
  float L = 0.0f, o = 0.0f;
  for (int s = 0; s < nrec; ++s) {
    const float m = rec[(size_t)s * DECODE_REC];
    if (m == -INFINITY) continue;
    const float f = __expf(m - M);
    L += rec[(size_t)s * DECODE_REC + 1] * f;
    o += rec[(size_t)s * DECODE_REC + 2 + c] * f;
  }
  out[(size_t)row * D + c] = (uint16_t)f2h(o / L);
}

template <int BITS, int GQ>
static hipError_t launch_decode_t(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                                  const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                                  int n_buf_cap, uint16_t* out, float* partial, hipStream_t st) {
  const int nsplit = (k0.n + MFMA_TS - 1) / MFMA_TS;
  size_t lds = (size_t)mfma_layout<GQ>(BITS, dm.g, k0.rank, v0.rank, dm.ppm).total;
  if (lds < sizeof(TailSmem<GQ>)) lds = sizeof(TailSmem<GQ>);
  static size_t lds_allowed = 0;  // raised once per process and kernel instance
  if (lds > lds_allowed) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_split_kernel<BITS, GQ>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_allowed = lds;
  }
  dim3 grid(nsplit + 1, dm.B * dm.H);
  hipLaunchKernelGGL((decode_split_kernel<BITS, GQ>), grid, dim3(256), lds, st, dm, k0, v0, cs, q, Kbuf, Vbuf,
                     n_buf, n_buf_cap, partial);
  hipLaunchKernelGGL(decode_combine_kernel, dim3(dm.B * dm.Hq), dim3(128), 0, st, (const float*)partial,
                     nsplit + 1, out);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_decode_b(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                                  const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                                  int n_buf_cap, uint16_t* out, float* partial, hipStream_t st) {
  switch (dm.Hq / dm.H) {
    case 1: return launch_decode_t<BITS, 1>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
    case 2: return launch_decode_t<BITS, 2>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
    case 4: return launch_decode_t<BITS, 4>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
    case 8: return launch_decode_t<BITS, 8>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_decode(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                         const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                         int n_buf_cap, uint16_t* out, float* partial, hipStream_t st) {
  if (dm.bits == 2) return launch_decode_b<2>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
  return launch_decode_b<4>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, out, partial, st);
}

}  // namespace gear
