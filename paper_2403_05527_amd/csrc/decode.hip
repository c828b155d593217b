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
#include <atomic>
#include "gear_internal.h"
#include "gear_launch.h"
#include "decode_mfma.h"
#include "decode_tail.h"

namespace gear {

static_assert(MFMA_TS == DECODE_SPLIT, "split size is part of the workspace layout");

// grid (nsplit + ncb + 1, B*H_kv), block 256.  Blocks [0, nsplit): 512 prefill tokens each;
// blocks [nsplit, nsplit + ncb): four pieces of appended chunks each (one piece = up to 128
// rows of one chunk, pp pieces per chunk), through the same code as the prefill; the
// last block: the fp16 streaming-buffer rows.
template <int BITS, int GQ, int LG>
__global__ __launch_bounds__(256, (GQ == 8 ? 3 : (BITS == 2 && (GQ <= 2 || (GQ == 4 && LG >= 6))) ? 5 : 4)) void decode_split_kernel(Dims dm, SegView k0, SegView v0, ChunkSet cs,
                                                              const uint16_t* __restrict__ q,
                                                              const uint16_t* __restrict__ Kbuf,
                                                              const uint16_t* __restrict__ Vbuf, int n_buf,
                                                              int n_buf_cap, int nsplit, int pp, int rank_cap,
                                                              int odd_rank, int q_len, int causal,
                                                              float* __restrict__ partial) {
  GEAR_DYN_LDS(smem_raw);
  const int slab = blockIdx.y, split = blockIdx.x;
  const int nrec = (int)gridDim.x;
  const int b = slab / dm.H, h = slab - b * dm.H;
  float* rec_base = partial + (((size_t)b * dm.Hq + h * GQ) * nrec + split) * DECODE_REC;
  const int rec_stride = nrec * DECODE_REC;
  const uint16_t* qg = q + ((size_t)b * dm.Hq + h * GQ) * D;
  const int wave = GEAR_WAVE_UNIFORM((int)(threadIdx.x >> 6));
  if (split == nrec - 1) {
    buffer_block<GQ>(*reinterpret_cast<TailSmem<GQ>*>(smem_raw), qg, Kbuf + (size_t)slab * n_buf_cap * D,
                     Vbuf + (size_t)slab * n_buf_cap * D, n_buf, q_len, causal, rec_base, rec_stride);
    return;
  }
  // one call site: the prefill segment for every wave, or one chunk piece per wave
  // (piece i = 4 * (split - nsplit) + wave covers rows [128 * (i % pp), ...) of chunk i / pp)
  SegView kw_ = k0, vw_ = v0;
  int tw0 = split * MFMA_TS + WTOK * wave, nw = k0.n - tw0;
  if (split >= nsplit) {
    const int item = 4 * (split - nsplit) + wave;
    const int j = pp == 2 ? item >> 1 : item, part = item - j * pp;   // pp is 1 or 2
    int n_j = 0, r_j = 0;
    if (j < cs.n_chunks) {
      n_j = cs.n[j];
      r_j = cs.rank[j];
    }
    kw_ = chunk_view(cs.k0, cs.stride, j < cs.n_chunks ? j : 0, n_j, r_j);
    vw_ = chunk_view(cs.v0, cs.stride, j < cs.n_chunks ? j : 0, n_j, r_j);
    tw0 = WTOK * part;
    nw = n_j - tw0;
  }
  mfma_block<BITS, GQ, LG>(smem_raw, dm, kw_, vw_, qg, slab, b, tw0, nw, k0.rank, v0.rank, rank_cap, odd_rank != 0, split < nsplit,
                           rec_base, rec_stride);
}

// grid (B*H_q), block 128: thread c merges channel c of the row's nrec records, 64 records per round.
// Lane s of every wave fetches (m, l) of record s, so the weights of up to 64 records come from one
// round of loads.  WIDE (rows with many records: long contexts at a small batch, where the kernel is a
// few blocks' latency): a thread requests its channel of all the round's records before anything is
// used, one load latency per round; otherwise eight at a time (fewer registers: more rows in flight).
// Records past the last read as 0 through the buffer view.
template <bool WIDE>
__global__ __launch_bounds__(128) void decode_combine_kernel(const float* __restrict__ partial, int nrec,
                                                             uint16_t* __restrict__ out) {
  const int row = blockIdx.x, c = threadIdx.x, lane = threadIdx.x & 63;
  const GEAR_BUF_T rb = GEAR_BUF_MAKE(partial + (size_t)row * nrec * DECODE_REC, nrec * (DECODE_REC * 4));
  float M = -INFINITY, L = 0.0f, o = 0.0f;
  for (int s0 = 0; s0 < nrec; s0 += 64) {
    const int cnt = nrec - s0 < 64 ? nrec - s0 : 64;
    const uint2 ml = GEAR_BUF_LOAD8(rb, (s0 + lane) * (DECODE_REC * 4));
    float v[WIDE ? 64 : 1];
    if constexpr (WIDE) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (16 * b < cnt) {   // block-uniform
#pragma unroll
          for (int u = 0; u < 16; ++u)
            v[16 * b + u] = __uint_as_float(GEAR_BUF_LOAD4(rb, ((s0 + 16 * b + u) * DECODE_REC + 2 + c) * 4));
        } else {
#pragma unroll
          for (int u = 0; u < 16; ++u) v[16 * b + u] = 0.0f;
        }
      }
    }
    const float m = lane < cnt ? __uint_as_float(ml.x) : -INFINITY;
    const float l = lane < cnt ? __uint_as_float(ml.y) : 0.0f;
    float Mn = m;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) Mn = fmaxf(Mn, __shfl_xor(Mn, d, 64));
    Mn = fmaxf(Mn, M);
    if (Mn == -INFINITY) continue;                      // nothing but empty records so far
    const float f = (m == -INFINITY) ? 0.0f : __expf(m - Mn);
    const float keep = (M == -INFINITY) ? 0.0f : __expf(M - Mn);
    L = L * keep + wave_sum_shfl(l * f);
    o *= keep;
    M = Mn;
    if constexpr (WIDE) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        if (16 * b < cnt) {
#pragma unroll
          for (int u = 0; u < 16; ++u) o += v[16 * b + u] * __shfl(f, 16 * b + u, 64);
        }
      }
    } else {
      constexpr int UN = 8;
      for (int j0 = 0; j0 < cnt; j0 += UN) {
        float w[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) w[u] = __uint_as_float(GEAR_BUF_LOAD4(rb, ((s0 + j0 + u) * DECODE_REC + 2 + c) * 4));
#pragma unroll
        for (int u = 0; u < UN; ++u) o += w[u] * __shfl(f, (j0 + u) & 63, 64);
      }
    }
  }
  out[(size_t)row * D + c] = (uint16_t)f2h(o / L);
}

template <int BITS, int GQ, int LG>
static hipError_t launch_decode_t(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                                  const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                                  int n_buf_cap, int rank_cap, int q_len, int causal, uint16_t* out, float* partial,
                                  hipStream_t st) {
  const int nsplit = (k0.n + MFMA_TS - 1) / MFMA_TS;
  const int pp = n_buf_cap > WTOK ? 2 : 1;            // pieces per chunk
  const int ncb = (cs.n_chunks * pp + 3) / 4;
  int rc = 0;                                         // largest rank of an appended chunk
  for (int j = 0; j < cs.n_chunks; ++j) rc = cs.rank[j] > rc ? cs.rank[j] : rc;
  if (rc > rank_cap) return hipErrorInvalidValue;     // the cache never stores more than its configured rank
  // a rank whose rows are not one 4-, 8- or 16-byte read anywhere in the launch
  auto one_read = [](int r) { return r == 0 || r == 2 || r == 4 || r == 8; };
  bool odd_rank = !one_read(k0.rank) || !one_read(v0.rank);
  for (int j = 0; j < cs.n_chunks; ++j) odd_rank = odd_rank || !one_read(cs.rank[j]);
  size_t lds = (size_t)mfma_layout<GQ>(BITS, dm.g, k0.rank, v0.rank, rc, dm.ppm, odd_rank).total;
  if (lds < sizeof(TailSmem<GQ>)) lds = sizeof(TailSmem<GQ>);
  static std::atomic<size_t> lds_allowed{0};  // raised once per process and kernel instance (two threads may both raise it: harmless)
  if (lds > lds_allowed.load(std::memory_order_relaxed)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_split_kernel<BITS, GQ, LG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_allowed.store(lds, std::memory_order_relaxed);
  }
  dim3 grid(nsplit + ncb + 1, dm.B * dm.H);
  hipLaunchKernelGGL((decode_split_kernel<BITS, GQ, LG>), grid, dim3(256), lds, st, dm, k0, v0, cs, q, Kbuf, Vbuf,
                     n_buf, n_buf_cap, nsplit, pp, rc, odd_rank ? 1 : 0, q_len, causal, partial);
  if (nsplit + ncb + 1 > 32)
    hipLaunchKernelGGL(decode_combine_kernel<true>, dim3(dm.B * dm.Hq), dim3(128), 0, st, (const float*)partial,
                       nsplit + ncb + 1, out);
  else
    hipLaunchKernelGGL(decode_combine_kernel<false>, dim3(dm.B * dm.Hq), dim3(128), 0, st, (const float*)partial,
                       nsplit + ncb + 1, out);
  return hipGetLastError();
}

template <int BITS>
static hipError_t launch_decode_b(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                                  const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                                  int n_buf_cap, int rank_cap, int q_len, int causal, uint16_t* out, float* partial,
                                  hipStream_t st) {
#define GEAR_DECODE_CASE(GQV)                                                                                          \
  case GQV:                                                                                                            \
    if (dm.g == 32) return launch_decode_t<BITS, GQV, 5>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, rank_cap, q_len, causal, out, partial, st); \
    if (dm.g == 64) return launch_decode_t<BITS, GQV, 6>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, rank_cap, q_len, causal, out, partial, st); \
    return launch_decode_t<BITS, GQV, 7>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, rank_cap, q_len, causal, out, partial, st);
  switch (dm.Hq / dm.H) {
    GEAR_DECODE_CASE(1)
    GEAR_DECODE_CASE(2)
    GEAR_DECODE_CASE(4)
    GEAR_DECODE_CASE(8)
    default: return hipErrorInvalidValue;
  }
#undef GEAR_DECODE_CASE
}

// q_len query rows per query head ([B, H_q, q_len, 128]): the rows of the query heads of one KV head lie
// next to each other, so they are run as (H_q / H) * q_len query columns of that KV head.
hipError_t launch_decode(const Dims& dm_in, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                         const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                         int n_buf_cap, int rank_cap, int q_len, int causal, uint16_t* out, float* partial,
                         hipStream_t st) {
  Dims dm = dm_in;
  dm.Hq = dm_in.Hq * q_len;
  if (dm.bits == 2)
    return launch_decode_b<2>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, rank_cap, q_len, causal, out, partial, st);
  return launch_decode_b<4>(dm, k0, v0, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, rank_cap, q_len, causal, out, partial, st);
}

}  // namespace gear
