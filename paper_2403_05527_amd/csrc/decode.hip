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
// the fp16 buffer with a plain-ALU path and an online softmax state.  Every
// block writes one partial record (m, l, o) per query head; decode_combine
// merges the records.
#include "gear_internal.h"
#include "gear_launch.h"
#include "decode_mfma.h"

namespace gear {

constexpr int TS = DECODE_TS;
static_assert(MFMA_TS == DECODE_SPLIT, "split size is part of the workspace layout");

template <int GQ>
struct DecodeSmem {
  float q[GQ][D];
  float sc[GQ][TS];
  float o_run[GQ][D];
  float o_tmp[GQ][D];
  float m_run[GQ], l_run[GQ];
  float qB[GQ][8], wv[GQ][8];
  float2 kd[9 * D];
  float2 vd[TS * 4];
  float red[GQ][4];
  float bc[GQ][2];
};

__device__ __forceinline__ SegView chunk_view(const SegView& base, uint64_t stride, int j, int n, int rank) {
  SegView v = base;
  const size_t off = (size_t)stride * j;
  v.codes = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.codes) + off);
  v.sz = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.sz) + off);
  v.A = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(base.A) + off);
  v.Bf = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(base.Bf) + off);
  v.sp_table = reinterpret_cast<uint2*>(reinterpret_cast<char*>(base.sp_table) + off);
  v.sp_pool = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.sp_pool) + off);
  v.n = n;
  v.rank = rank;
  return v;
}

// Merge `n_rows` new scores (in S.sc, unscaled) into the running softmax state:
// afterwards S.sc holds p_t = exp(s_t/sqrt(d) - m_run) and o_run is rescaled.
template <int GQ>
__device__ __forceinline__ void softmax_merge(DecodeSmem<GQ>& S, int n_rows) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float scale = 0.08838834764831845f;  // 1/sqrt(128)
  float s[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    s[hq] = tid < n_rows ? S.sc[hq][tid] * scale : -INFINITY;
    const float mx = wave_max(s[hq]);
    if (lane == 0) S.red[hq][wave] = mx;
  }
  __syncthreads();
  if (tid < GQ) {
    const float m_loc = fmaxf(fmaxf(S.red[tid][0], S.red[tid][1]), fmaxf(S.red[tid][2], S.red[tid][3]));
    const float m_old = S.m_run[tid];
    const float m_new = fmaxf(m_old, m_loc);
    S.bc[tid][0] = m_new;
    S.bc[tid][1] = (m_old == -INFINITY) ? 0.0f : __expf(m_old - m_new);
  }
  __syncthreads();
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    const float p = tid < n_rows ? __expf(s[hq] - S.bc[hq][0]) : 0.0f;
    if (tid < n_rows) S.sc[hq][tid] = p;
    const float sum = wave_sum(p);
    if (lane == 0) S.red[hq][wave] = sum;
  }
  for (int i = tid; i < GQ * D; i += 256) S.o_run[i / D][i % D] *= S.bc[i / D][1];
  __syncthreads();
  if (tid < GQ) {
    S.l_run[tid] = S.l_run[tid] * S.bc[tid][1] + (S.red[tid][0] + S.red[tid][1] + S.red[tid][2] + S.red[tid][3]);
    S.m_run[tid] = S.bc[tid][0];
  }
  __syncthreads();
}

// Tokens [t_begin, t_end) of one compressed segment; t_end - t_begin <= TS and
// t_begin is a multiple of TS.
template <int GQ>
__device__ void attend_range(DecodeSmem<GQ>& S, const Dims& dm, const SegView& ks, const SegView& vs,
                             int slab, int b, int t_begin, int t_end) {
  const int tid = threadIdx.x;
  const int nr = t_end - t_begin;
  const int g = dm.g, bits = dm.bits;
  const uint32_t cmask = (1u << bits) - 1u;
  const int per = 32 / bits;
  const int rk = ks.rank;

  // q^T B_K (down-projection), group parameters of the range
  if (tid < GQ * 8) {
    const int hq = tid >> 3, r = tid & 7;
    float s = 0.0f;
    if (r < rk)
      for (int c = 0; c < D; ++c) s += S.q[hq][c] * h2f(ks.Bf[((size_t)slab * D + c) * rk + r]);
    S.qB[hq][r] = s;
  }
  const int grp0 = t_begin / g;
  const int ngl = (nr + g - 1) / g;
  for (int i = tid; i < ngl * D; i += 256) {
    const uint32_t sb = ks.sz[((size_t)slab * ks.ng_cap + grp0) * D + i];
    S.kd[i] = make_float2(h2f(sb & 0xFFFFu), h2f(sb >> 16));
  }
  const int ngv = D / g;
  for (int i = tid; i < nr * ngv; i += 256) {
    const uint32_t sb = vs.sz[((size_t)slab * vs.n_cap + t_begin) * ngv + i];
    S.vd[i] = make_float2(h2f(sb & 0xFFFFu), h2f(sb >> 16));
  }
  __syncthreads();

  // ---- scores from the quantized backbone + low-rank term
  if (tid < nr) {
    const int t = t_begin + tid;
    const uint32_t* row = ks.codes + ((size_t)slab * ks.n_cap + t) * dm.wpr;
    const float2* kd = S.kd + (size_t)(tid / g) * D;
    float s[GQ];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) s[hq] = 0.0f;
    for (int wi = 0; wi < dm.wpr; wi += 4) {
      const uint4 w4 = *reinterpret_cast<const uint4*>(row + wi);
      const uint32_t ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        for (int i = 0; i < per; ++i) {
          const int c = (wi + j) * per + i;
          const float2 dz = kd[c];
          const float kv = (float)((ww[j] >> (i * bits)) & cmask) * dz.x + dz.y;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) s[hq] += S.q[hq][c] * kv;
        }
      }
    }
    for (int r = 0; r < rk; ++r) {
      const float a = h2f(ks.A[((size_t)slab * ks.n_cap + t) * rk + r]);
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) s[hq] += S.qB[hq][r] * a;
    }
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) S.sc[hq][tid] = s[hq];
  }
  __syncthreads();

  // ---- sparse Key term: lists ordered (t, c); the first entry of a token sums the token's run
  const int tile0 = t_begin / TILE, tile1 = (t_end + TILE - 1) / TILE;
  if (dm.ppm > 0) {
    for (int tile = tile0; tile < tile1; ++tile) {
      const uint2 oc = ks.sp_table[(size_t)slab * ks.ntile_cap + tile];
      const uint32_t* lst = ks.sp_pool + (size_t)slab * ks.pool_cap + oc.x;
      for (uint32_t e = tid; e < oc.y; e += 256) {
        const uint32_t me = lst[e];
        const uint32_t tl = (me & 0xFFFFu) >> 7;
        if (e > 0 && ((lst[e - 1] & 0xFFFFu) >> 7) == tl) continue;
        float acc[GQ];
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) acc[hq] = 0.0f;
        for (uint32_t f = e; f < oc.y; ++f) {
          const uint32_t en = lst[f];
          if (((en & 0xFFFFu) >> 7) != tl) break;
          const float v = h2f(en >> 16);
          const int c = en & 127u;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) acc[hq] += S.q[hq][c] * v;
        }
        const int row = tile * TILE + (int)tl - t_begin;
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) S.sc[hq][row] += acc[hq];
      }
    }
    __syncthreads();
  }

  softmax_merge<GQ>(S, nr);

  // ---- Value side: quantized backbone
  {
    const int c = tid & 127, half = tid >> 7;
    const int tpw = dm.tpw;
    const int ntg = (nr + tpw - 1) / tpw;
    const int G = c / g;
    float o[GQ];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) o[hq] = 0.0f;
    for (int tg = half; tg < ntg; tg += 2) {
      const int tgg = t_begin / tpw + tg;
      const uint32_t w =
          vs.codes[((size_t)slab * vs.nblk_cap + (tgg >> 2)) * 512 + ((tgg & 3) * 16 + (c & 15)) * 8 + (c >> 4)];
      for (int i = 0; i < tpw; ++i) {
        const int tl = tg * tpw + i;
        if (tl < nr) {
          const float2 dz = S.vd[tl * ngv + G];
          const float v = (float)((w >> (i * bits)) & cmask) * dz.x + dz.y;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][tl] * v;
        }
      }
    }
    if (half == 1) {
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) S.o_tmp[hq][c] = o[hq];
    }
    // p^T A_V (down-projection)
    const int rv = vs.rank;
    if (tid < GQ * 8) {
      const int hq = tid >> 3, r = tid & 7;
      float s = 0.0f;
      if (r < rv)
        for (int tl = 0; tl < nr; ++tl)
          s += S.sc[hq][tl] * h2f(vs.A[((size_t)slab * vs.n_cap + t_begin + tl) * rv + r]);
      S.wv[hq][r] = s;
    }
    __syncthreads();
    if (half == 0) {
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) {
        float acc = o[hq] + S.o_tmp[hq][c];
        for (int r = 0; r < rv; ++r) acc += S.wv[hq][r] * h2f(vs.Bf[((size_t)slab * D + c) * rv + r]);
        S.o_run[hq][c] += acc;
      }
    }
    __syncthreads();
  }

  // ---- sparse Value term: lists ordered (c, t); the first entry of a channel sums the channel's run
  if (dm.ppm > 0) {
    for (int tile = tile0; tile < tile1; ++tile) {
      const uint2 oc = vs.sp_table[(size_t)slab * vs.ntile_cap + tile];
      const uint32_t* lst = vs.sp_pool + (size_t)b * vs.pool_cap + oc.x;
      for (uint32_t e = tid; e < oc.y; e += 256) {
        const uint32_t me = lst[e];
        const uint32_t ch = me & 127u;
        if (e > 0 && (lst[e - 1] & 127u) == ch) continue;
        float acc[GQ];
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) acc[hq] = 0.0f;
        for (uint32_t f = e; f < oc.y; ++f) {
          const uint32_t en = lst[f];
          if ((en & 127u) != ch) break;
          const float v = h2f(en >> 16);
          const int row = tile * TILE + (int)((en & 0xFFFFu) >> 7) - t_begin;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) acc[hq] += S.sc[hq][row] * v;
        }
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) S.o_run[hq][ch] += acc[hq];
      }
      __syncthreads();
    }
  }
}

// The first n_buf rows of the fp16 streaming buffer (n_buf <= TS).
template <int GQ>
__device__ void attend_buffer(DecodeSmem<GQ>& S, const uint16_t* Kb, const uint16_t* Vb, int n_buf) {
  const int tid = threadIdx.x;
  if (tid < n_buf) {
    float s[GQ];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) s[hq] = 0.0f;
    const uint4* row = reinterpret_cast<const uint4*>(Kb + (size_t)tid * D);
    for (int i = 0; i < D / 8; ++i) {
      const uint4 v = row[i];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float kv = h2f((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) s[hq] += S.q[hq][i * 8 + e] * kv;
      }
    }
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) S.sc[hq][tid] = s[hq];
  }
  __syncthreads();
  softmax_merge<GQ>(S, n_buf);
  const int c = tid & 127, half = tid >> 7;
  float o[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) o[hq] = 0.0f;
  for (int r = half; r < n_buf; r += 2) {
    const float v = h2f(Vb[(size_t)r * D + c]);
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][r] * v;
  }
  if (half == 1) {
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) S.o_tmp[hq][c] = o[hq];
  }
  __syncthreads();
  if (half == 0) {
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) S.o_run[hq][c] += o[hq] + S.o_tmp[hq][c];
  }
  __syncthreads();
}

// Chunk segments and the fp16 buffer: the generic (plain ALU) path with a running
// softmax state.  One block per (b, h_kv).
template <int GQ>
__device__ void tail_block(DecodeSmem<GQ>& S, const Dims& dm, const ChunkSet& cs, const uint16_t* __restrict__ q,
                           const uint16_t* __restrict__ Kbuf, const uint16_t* __restrict__ Vbuf, int n_buf,
                           int n_buf_cap, int slab, float* __restrict__ rec_base, int rec_stride) {
  const int b = slab / dm.H, h = slab - b * dm.H;
  const int tid = threadIdx.x;
  for (int i = tid; i < GQ * D; i += 256) {
    const int hq = i / D, c = i % D;
    S.q[hq][c] = h2f(q[((size_t)b * dm.Hq + h * GQ + hq) * D + c]);
    S.o_run[hq][c] = 0.0f;
  }
  if (tid < GQ) {
    S.m_run[tid] = -INFINITY;
    S.l_run[tid] = 0.0f;
  }
  __syncthreads();
  for (int j = 0; j < cs.n_chunks; ++j) {
    const SegView kj = chunk_view(cs.k0, cs.stride, j, cs.n[j], cs.rank[j]);
    const SegView vj = chunk_view(cs.v0, cs.stride, j, cs.n[j], cs.rank[j]);
    attend_range<GQ>(S, dm, kj, vj, slab, b, 0, cs.n[j]);
  }
  if (n_buf > 0)
    attend_buffer<GQ>(S, Kbuf + (size_t)slab * n_buf_cap * D, Vbuf + (size_t)slab * n_buf_cap * D, n_buf);
  for (int i = tid; i < GQ * D; i += 256) {
    const int hq = i / D, c = i % D;
    float* rec = rec_base + (size_t)hq * rec_stride;
    rec[2 + c] = S.o_run[hq][c];
    if (c == 0) {
      rec[0] = S.m_run[hq];
      rec[1] = S.l_run[hq];
    }
  }
}

// grid (nsplit + 1, B*H_kv), block 256.  Blocks 0..nsplit-1: MFMA_TS prefill
// tokens each (MFMA path); block nsplit: chunks + buffer.
// Dynamic LDS: MfmaSmem<GQ> | 4 x opnd_halfs fp16 (per-wave operand staging,
// reused for the cross-wave reduction), or DecodeSmem<GQ> for the tail block.
template <int BITS, int GQ>
__global__ __launch_bounds__(256, 4) void decode_split_kernel(Dims dm, SegView k0, SegView v0, ChunkSet cs,
                                                           const uint16_t* __restrict__ q,
                                                           const uint16_t* __restrict__ Kbuf,
                                                           const uint16_t* __restrict__ Vbuf, int n_buf,
                                                           int n_buf_cap, float* __restrict__ partial,
                                                           int opnd_halfs) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int slab = blockIdx.y, split = blockIdx.x;
  const int nsplit = (int)gridDim.x - 1;
  const int b = slab / dm.H, h = slab - b * dm.H;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float* rec_base = partial + (((size_t)b * dm.Hq + h * GQ) * (nsplit + 1) + split) * DECODE_REC;
  const int rec_stride = (nsplit + 1) * DECODE_REC;
  if (split == nsplit) {
    tail_block<GQ>(*reinterpret_cast<DecodeSmem<GQ>*>(smem_raw), dm, cs, q, Kbuf, Vbuf, n_buf, n_buf_cap, slab,
                   rec_base, rec_stride);
    return;
  }

  MfmaSmem<GQ>& S = *reinterpret_cast<MfmaSmem<GQ>*>(smem_raw);
  constexpr size_t kOpndOff = (sizeof(MfmaSmem<GQ>) + 15) & ~size_t(15);
  _Float16* opnd_all = reinterpret_cast<_Float16*>(smem_raw + kOpndOff);
  _Float16* opnd = opnd_all + (size_t)wave * opnd_halfs;
  const int t_begin = split * MFMA_TS;
  const int t_end = min(k0.n, t_begin + MFMA_TS);
  const int nr = t_end - t_begin;
  const int rk = k0.rank, rv = v0.rank;
  const float scale = 0.08838834764831845f;  // 1/sqrt(128)

  for (int i = tid; i < GQ * D; i += 256) {
    const int hq = i / D, c = i % D;
    S.q[hq][c] = h2f(q[((size_t)b * dm.Hq + h * GQ + hq) * D + c]);
    S.o_fin[hq][c] = 0.0f;
  }
  __syncthreads();
  if (tid < GQ * 8) {  // q^T B_K
    const int hq = tid >> 3, r = tid & 7;
    float s = 0.0f;
    if (r < rk)
      for (int c = 0; c < D; ++c) s += S.q[hq][c] * h2f(k0.Bf[((size_t)slab * D + c) * rk + r]);
    S.qB[hq][r] = s;
  }

  mfma_key_scores<BITS, GQ>(S, opnd, dm, k0, slab, t_begin, t_end);  // ends with a block barrier

  // low-rank Key term, one token per thread
  for (int tl = tid; tl < nr; tl += 256) {
    float a[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) a[r] = r < rk ? h2f(k0.A[((size_t)slab * k0.n_cap + t_begin + tl) * rk + r]) : 0.0f;
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      float s = S.sc[hq][tl];
#pragma unroll
      for (int r = 0; r < 8; ++r) s += S.qB[hq][r] * a[r];
      S.sc[hq][tl] = s;
    }
  }
  __syncthreads();
  // sparse Key term (lists ordered (t, c): the first entry of a token sums the token's run)
  const int tile0 = t_begin / TILE, tile1 = (t_end + TILE - 1) / TILE;
  if (dm.ppm > 0) {
    for (int tile = tile0; tile < tile1; ++tile) {
      const uint2 oc = k0.sp_table[(size_t)slab * k0.ntile_cap + tile];
      const uint32_t* lst = k0.sp_pool + (size_t)slab * k0.pool_cap + oc.x;
      for (uint32_t e = tid; e < oc.y; e += 256) {
        const uint32_t me = lst[e];
        const uint32_t tl = (me & 0xFFFFu) >> 7;
        if (e > 0 && ((lst[e - 1] & 0xFFFFu) >> 7) == tl) continue;
        float acc[GQ];
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) acc[hq] = 0.0f;
        for (uint32_t f = e; f < oc.y; ++f) {
          const uint32_t en = lst[f];
          if (((en & 0xFFFFu) >> 7) != tl) break;
          const float v = h2f(en >> 16);
          const int c = en & 127u;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) acc[hq] += S.q[hq][c] * v;
        }
        const int row = tile * TILE + (int)tl - t_begin;
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) S.sc[hq][row] += acc[hq];
      }
    }
    __syncthreads();
  }

  // block-local softmax: m, p = exp(s - m), l
  {
    float s0[GQ], s1[GQ];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      s0[hq] = tid < nr ? S.sc[hq][tid] * scale : -INFINITY;
      s1[hq] = tid + 256 < nr ? S.sc[hq][tid + 256] * scale : -INFINITY;
      const float mx = wave_max(fmaxf(s0[hq], s1[hq]));
      if (lane == 0) S.red[hq][wave] = mx;
    }
    __syncthreads();
    if (tid < GQ)
      S.stat[tid][0] = fmaxf(fmaxf(S.red[tid][0], S.red[tid][1]), fmaxf(S.red[tid][2], S.red[tid][3]));
    __syncthreads();
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      const float m = S.stat[hq][0];
      const float p0 = tid < nr ? __expf(s0[hq] - m) : 0.0f;
      const float p1 = tid + 256 < nr ? __expf(s1[hq] - m) : 0.0f;
      if (tid < nr) S.sc[hq][tid] = p0;
      if (tid + 256 < nr) S.sc[hq][tid + 256] = p1;
      const float sum = wave_sum(p0 + p1);
      if (lane == 0) S.red[hq][wave] = sum;
    }
    __syncthreads();
    if (tid < GQ) S.stat[tid][1] = S.red[tid][0] + S.red[tid][1] + S.red[tid][2] + S.red[tid][3];
  }

  floatx4 acc[8];
  mfma_value_accum<BITS, GQ>(S, opnd, dm, v0, slab, t_begin, t_end, acc);  // ends with a block barrier

  // p^T A_V (down-projection): per-thread partials over its tokens, then block sums
  {
    float part[GQ][8];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
      for (int r = 0; r < 8; ++r) part[hq][r] = 0.0f;
    for (int tl = tid; tl < nr; tl += 256) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        if (r < rv) {
          const float a = h2f(v0.A[((size_t)slab * v0.n_cap + t_begin + tl) * rv + r]);
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) part[hq][r] += S.sc[hq][tl] * a;
        }
      }
    }
    float* wred = reinterpret_cast<float*>(opnd_all);  // [4][GQ][8], staging area is free now
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq)
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const float s = r < rv ? wave_sum(part[hq][r]) : 0.0f;
        if (lane == 0) wred[(wave * GQ + hq) * 8 + r] = s;
      }
    __syncthreads();
    if (tid < GQ * 8)
      S.wv[tid >> 3][tid & 7] = wred[tid] + wred[GQ * 8 + tid] + wred[2 * GQ * 8 + tid] + wred[3 * GQ * 8 + tid];
    __syncthreads();
  }
  // sparse Value term (lists ordered (c, t): the first entry of a channel sums the channel's run)
  if (dm.ppm > 0) {
    for (int tile = tile0; tile < tile1; ++tile) {
      const uint2 oc = v0.sp_table[(size_t)slab * v0.ntile_cap + tile];
      const uint32_t* lst = v0.sp_pool + (size_t)b * v0.pool_cap + oc.x;
      for (uint32_t e = tid; e < oc.y; e += 256) {
        const uint32_t me = lst[e];
        const uint32_t ch = me & 127u;
        if (e > 0 && (lst[e - 1] & 127u) == ch) continue;
        float a2[GQ];
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) a2[hq] = 0.0f;
        for (uint32_t f = e; f < oc.y; ++f) {
          const uint32_t en = lst[f];
          if ((en & 127u) != ch) break;
          const float v = h2f(en >> 16);
          const int row = tile * TILE + (int)((en & 0xFFFFu) >> 7) - t_begin;
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) a2[hq] += S.sc[hq][row] * v;
        }
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) S.o_fin[hq][ch] += a2[hq];
      }
      __syncthreads();
    }
  }
  // cross-wave reduction of the MFMA accumulators through the (now free) staging area
  {
    float* opart = reinterpret_cast<float*>(opnd_all);  // [4][GQ][D]
    const int n16 = lane & 15, kg = lane >> 4;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int hq0 = 2 * kg, hq1 = 2 * kg + 1;
      if (hq0 < GQ) opart[((size_t)wave * GQ + hq0) * D + 16 * j + n16] = (acc[j][0] + acc[j][1]) * MFMA_OUT_SCALE;
      if (hq1 < GQ) opart[((size_t)wave * GQ + hq1) * D + 16 * j + n16] = (acc[j][2] + acc[j][3]) * MFMA_OUT_SCALE;
    }
    __syncthreads();
    const int NG = D / dm.g;
    for (int i = tid; i < GQ * D; i += 256) {
      const int hq = i / D, c = i % D, G = c / dm.g;
      float o = S.o_fin[hq][c];
#pragma unroll
      for (int w = 0; w < 4; ++w) o += opart[((size_t)w * GQ + hq) * D + c] + S.pm[w][hq][G];
      for (int r = 0; r < rv; ++r) o += S.wv[hq][r] * h2f(v0.Bf[((size_t)slab * D + c) * rv + r]);
      float* rec = rec_base + (size_t)hq * rec_stride;
      rec[2 + c] = o;
      if (c == 0) {
        rec[0] = S.stat[hq][0];
        rec[1] = S.stat[hq][1];
      }
    }
    (void)NG;
  }
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

int decode_nsplit(int n_prefill) { return (n_prefill + MFMA_TS - 1) / MFMA_TS; }

template <int BITS, int GQ>
static hipError_t launch_decode_t(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                                  const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                                  int n_buf_cap, uint16_t* out, float* partial, hipStream_t st) {
  const int nsplit = decode_nsplit(k0.n);
  const int TB = BITS == 2 ? 64 : 32;
  int opnd_halfs = (D / dm.g) * 16 * TB;
  if (opnd_halfs < 16 * D) opnd_halfs = 16 * D;
  size_t lds = ((sizeof(MfmaSmem<GQ>) + 15) & ~size_t(15)) + (size_t)4 * opnd_halfs * 2;
  if (lds < sizeof(DecodeSmem<GQ>)) lds = sizeof(DecodeSmem<GQ>);
  static size_t lds_allowed = 0;  // raised once per process and kernel instance
  if (lds > lds_allowed) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_split_kernel<BITS, GQ>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    lds_allowed = lds;
  }
  dim3 grid(nsplit + 1, dm.B * dm.H);
  hipLaunchKernelGGL((decode_split_kernel<BITS, GQ>), grid, dim3(256), lds, st, dm, k0, v0, cs, q, Kbuf, Vbuf,
                     n_buf, n_buf_cap, partial, opnd_halfs);
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
