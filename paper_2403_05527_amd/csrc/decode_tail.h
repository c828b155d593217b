// Attention over the appended chunk segments and the fp16 streaming buffer for
// one (b, h_kv): a plain-ALU path.  The rows of several chunks (each with its own
// quantization groups, low-rank factors and outlier lists) and the buffer rows
// are laid side by side and processed as ONE pass of up to TAIL_ROWS rows, so the
// number of dependent memory round trips does not grow with the number of
// chunks; an online softmax state carries over when more passes are needed.
#pragma once
#include "gear_internal.h"
#include "gear_launch.h"

namespace gear {

constexpr int TAIL_ROWS = 256;   // rows per pass (one per thread)
constexpr int TAIL_CHUNKS = 32;  // chunk segments per pass

template <int GQ>
struct TailSmem {
  float q[GQ][D];
  float sc[GQ][TAIL_ROWS];
  float o_run[GQ][D];
  float o_half[2][GQ][D];
  float osp[4][GQ][D];
  float m_run[GQ], l_run[GQ];
  float red[GQ][4];
  float bc[GQ][2];
  float2 vd[TAIL_ROWS * 4];
  float qB[TAIL_CHUNKS][GQ][8];
  float wv[TAIL_CHUNKS][GQ][8];
  uint2 tabk[TAIL_CHUNKS][4], tabv[TAIL_CHUNKS][4];
  int row0[TAIL_CHUNKS + 1];
  short row_chunk[TAIL_ROWS];
  short row_tok[TAIL_ROWS];
  int plan[4];  // npc, nrows (chunk rows), nbuf_rows, unused
};

__device__ __forceinline__ SegView chunk_view(const SegView& base, uint64_t stride, int j, int n, int rank) {
  SegView v = base;
  const size_t off = (size_t)stride * j;
  v.codes = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.codes) + off);
  v.sz = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.sz) + off);
  v.A = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(base.A) + off);
  v.Bf = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(base.Bf) + off);
  v.ell = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.ell) + off);
  v.sp_table = reinterpret_cast<uint2*>(reinterpret_cast<char*>(base.sp_table) + off);
  v.sp_pool = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(base.sp_pool) + off);
  v.n = n;
  v.rank = rank;
  return v;
}

// Merge n_rows new raw scores (S.sc) into the running softmax state: afterwards
// S.sc holds p_t = exp(s_t / sqrt(d) - m_run) and o_run is rescaled.
template <int GQ>
__device__ __forceinline__ void tail_softmax_merge(TailSmem<GQ>& S, int n_rows) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float scale = 0.08838834764831845f;  // 1/sqrt(128)
  float s[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    s[hq] = tid < n_rows ? S.sc[hq][tid] * scale : -INFINITY;
    const float mx = wave_max(s[hq]);
    if (lane == 0) S.red[hq][wave] = mx;
  }
  block_lds_sync();
  if (tid < GQ) {
    const float m_loc = fmaxf(fmaxf(S.red[tid][0], S.red[tid][1]), fmaxf(S.red[tid][2], S.red[tid][3]));
    const float m_old = S.m_run[tid];
    const float m_new = fmaxf(m_old, m_loc);
    S.bc[tid][0] = m_new;
    S.bc[tid][1] = (m_old == -INFINITY) ? 0.0f : __expf(m_old - m_new);
  }
  block_lds_sync();
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    const float p = tid < n_rows ? __expf(s[hq] - S.bc[hq][0]) : 0.0f;
    S.sc[hq][tid] = p;
    const float sum = wave_sum(p);
    if (lane == 0) S.red[hq][wave] = sum;
  }
  for (int i = tid; i < GQ * D; i += 256) S.o_run[i / D][i % D] *= S.bc[i / D][1];
  block_lds_sync();
  if (tid < GQ) {
    S.l_run[tid] = S.l_run[tid] * S.bc[tid][1] + (S.red[tid][0] + S.red[tid][1] + S.red[tid][2] + S.red[tid][3]);
    S.m_run[tid] = S.bc[tid][0];
  }
  block_lds_sync();
}

template <int GQ>
__device__ void tail_block(TailSmem<GQ>& S, const Dims& dm, const ChunkSet& cs, const uint16_t* __restrict__ qg,
                           const uint16_t* __restrict__ Kb, const uint16_t* __restrict__ Vb, int n_buf, int slab,
                           int b, float* __restrict__ rec_base, int rec_stride) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int g = dm.g, bits = dm.bits, tpw = dm.tpw, NG = D / g;
  const uint32_t cmask = (1u << bits) - 1u;
  const int per = 32 / bits;
  for (int i = tid; i < GQ * D; i += 256) {
    S.q[i / D][i % D] = h2f(qg[i]);
    S.o_run[i / D][i % D] = 0.0f;
  }
  if (tid < GQ) {
    S.m_run[tid] = -INFINITY;
    S.l_run[tid] = 0.0f;
  }
  int j_next = 0, buf_done = 0;
  // block-uniform loop; every pass consumes at least one chunk or one buffer row
  for (int pass = 0; pass < 2 * GEAR_MAX_CHUNKS && (j_next < cs.n_chunks || buf_done < n_buf); ++pass) {
    block_lds_sync();
    // ---- plan the pass (every thread computes the same plan)
    int npc = 0, nrows = 0;
    while (j_next + npc < cs.n_chunks && npc < TAIL_CHUNKS && nrows + cs.n[j_next + npc] <= TAIL_ROWS) {
      nrows += cs.n[j_next + npc];
      ++npc;
    }
    int nbuf_rows = 0;
    if (j_next + npc == cs.n_chunks) {
      nbuf_rows = n_buf - buf_done;
      if (nbuf_rows > TAIL_ROWS - nrows) nbuf_rows = TAIL_ROWS - nrows;
    }
    const int jbase = j_next, bbase = buf_done;
    const int ntot = nrows + nbuf_rows;
    if (tid == 0) {
      int run = 0;
      for (int jc = 0; jc < npc; ++jc) { S.row0[jc] = run; run += cs.n[jbase + jc]; }
      S.row0[npc] = run;
    }
    for (int i = tid; i < 4 * GQ * D; i += 256) (&S.osp[0][0][0])[i] = 0.0f;
    block_lds_sync();
    // ---- row map, per-chunk tables, q^T B_K, Value (scale, zero) of every row
    for (int jc = tid; jc < npc; jc += 256) {
      const int n_j = cs.n[jbase + jc], r0 = S.row0[jc];
      for (int i = 0; i < n_j; ++i) { S.row_chunk[r0 + i] = (short)jc; S.row_tok[r0 + i] = (short)i; }
    }
    for (int k = tid; k < nbuf_rows; k += 256) { S.row_chunk[nrows + k] = -1; S.row_tok[nrows + k] = (short)(bbase + k); }
    if (dm.ppm > 0) {
      for (int i = tid; i < npc * 8; i += 256) {
        const int jc = i >> 3, which = (i >> 2) & 1, tile = i & 3;
        const int j = jbase + jc, n_j = cs.n[j];
        uint2 e = make_uint2(0, 0);
        if (tile * TILE < n_j) {
          const SegView v = chunk_view(which ? cs.v0 : cs.k0, cs.stride, j, n_j, cs.rank[j]);
          e = v.sp_table[(size_t)slab * v.ntile_cap + tile];
          if (e.x > v.pool_cap) e.x = v.pool_cap;   // a table entry is trusted only as far as its pool reaches
          if (e.y > v.pool_cap - e.x) e.y = v.pool_cap - e.x;
        }
        if (which) S.tabv[jc][tile] = e; else S.tabk[jc][tile] = e;
      }
    }
    for (int i = tid; i < npc * GQ * 8; i += 256) {
      const int jc = i / (GQ * 8), hq = (i >> 3) % GQ, r = i & 7;
      const int j = jbase + jc, rk = cs.rank[j];
      float s = 0.0f;
      if (r < rk) {
        const SegView kv = chunk_view(cs.k0, cs.stride, j, cs.n[j], rk);
        for (int c = 0; c < D; ++c) s += S.q[hq][c] * h2f(kv.Bf[((size_t)slab * D + c) * rk + r]);
      }
      S.qB[jc][hq][r] = s;
    }
    block_lds_sync();
    if (tid < nrows) {
      const int jc = S.row_chunk[tid], t = S.row_tok[tid], j = jbase + jc;
      const SegView vv = chunk_view(cs.v0, cs.stride, j, cs.n[j], cs.rank[j]);
      for (int G = 0; G < NG; ++G) {
        const uint32_t sb = vv.sz[((size_t)slab * vv.n_cap + t) * NG + G];
        S.vd[tid * NG + G] = make_float2(h2f(sb & 0xFFFFu), h2f(sb >> 16));
      }
    }
    // ---- raw scores, one row per thread
    if (tid < ntot) {
      float s[GQ];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) s[hq] = 0.0f;
      const int jc = S.row_chunk[tid], t = S.row_tok[tid];
      if (jc >= 0) {
        const int j = jbase + jc, rk = cs.rank[j];
        const SegView kv = chunk_view(cs.k0, cs.stride, j, cs.n[j], rk);
        const uint32_t* row = kv.codes + ((size_t)slab * kv.n_cap + t) * dm.wpr;
        const uint32_t* szr = kv.sz + ((size_t)slab * kv.ng_cap + t / g) * D;
        for (int wi = 0; wi < dm.wpr; ++wi) {
          const uint32_t w = row[wi];
          for (int i4 = 0; i4 < per; i4 += 4) {
            const uint4 s4 = *reinterpret_cast<const uint4*>(szr + wi * per + i4);
            const uint32_t sb[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int c = wi * per + i4 + e;
              const float kvv = (float)((w >> ((i4 + e) * bits)) & cmask) * h2f(sb[e] & 0xFFFFu) + h2f(sb[e] >> 16);
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) s[hq] += S.q[hq][c] * kvv;
            }
          }
        }
        for (int r = 0; r < rk; ++r) {
          const float a = h2f(kv.A[((size_t)slab * kv.n_cap + t) * rk + r]);
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) s[hq] += S.qB[jc][hq][r] * a;
        }
        if (dm.ppm > 0) {  // the row's fixed outlier slots (an empty slot is channel 0 with value +0)
          const uint4 e4 = *reinterpret_cast<const uint4*>(kv.ell + ((size_t)slab * kv.n_cap + t) * ELL_K);
          const uint32_t es[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
          for (int i = 0; i < ELL_K; ++i) {
            const float v = h2f(es[i] >> 16);
            const int c = es[i] & 127u;
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) s[hq] += S.q[hq][c] * v;
          }
        }
      } else {
        const uint4* row = reinterpret_cast<const uint4*>(Kb + (size_t)t * D);
        for (int i = 0; i < D / 8; ++i) {
          const uint4 v = row[i];
          const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float kvv = h2f((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) s[hq] += S.q[hq][i * 8 + e] * kvv;
          }
        }
      }
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) S.sc[hq][tid] = s[hq];
    }
    block_lds_sync();
    // ---- sparse Key term: wave w takes chunks w, w+4, ...; lists ordered (t, c)
    if (dm.ppm > 0) {
      for (int jc = wave; jc < npc; jc += 4) {
        const int j = jbase + jc, n_j = cs.n[j];
        const SegView kv = chunk_view(cs.k0, cs.stride, j, n_j, cs.rank[j]);
        for (int tile = 0; tile * TILE < n_j; ++tile) {
          const uint2 oc = S.tabk[jc][tile];
          const uint32_t* lst = kv.sp_pool + (size_t)slab * kv.pool_cap + oc.x;
          for (uint32_t e = lane; e < oc.y; e += 64) {
            const uint32_t me = lst[e];
            const uint32_t tl = (me & 0xFFFFu) >> 7;
            if (e > 0 && ((lst[e - 1] & 0xFFFFu) >> 7) == tl) continue;
            float a2[GQ];
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) a2[hq] = 0.0f;
            for (uint32_t f = e; f < oc.y; ++f) {
              const uint32_t en = lst[f];
              if (((en & 0xFFFFu) >> 7) != tl) break;
              const float v = h2f(en >> 16);
              const int c = en & 127u;
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) a2[hq] += S.q[hq][c] * v;
            }
            const int row = S.row0[jc] + tile * TILE + (int)tl;
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) S.sc[hq][row] += a2[hq];
          }
        }
      }
      block_lds_sync();
    }

    tail_softmax_merge<GQ>(S, ntot);

    // ---- Value side: thread (channel c, half) walks chunks half, half+2, ... and buffer rows
    {
      const int c = tid & 127, half = tid >> 7, G = c / g;
      float o[GQ];
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) o[hq] = 0.0f;
      for (int jc = half; jc < npc; jc += 2) {
        const int j = jbase + jc, n_j = cs.n[j], r0 = S.row0[jc];
        const SegView vv = chunk_view(cs.v0, cs.stride, j, n_j, cs.rank[j]);
        if (dm.ppm > 0) {  // the channel's fixed outlier slots of every tile (empty: row 0, value +0)
          for (int tile = 0; tile * TILE < n_j; ++tile) {
            const uint2 ev = *reinterpret_cast<const uint2*>(vv.ell + (((size_t)slab * vv.ntile_cap + tile) * D + c) * ELL_V);
            const uint32_t es[2] = {ev.x, ev.y};
#pragma unroll
            for (int i = 0; i < ELL_V; ++i) {
              const float v = h2f(es[i] >> 16);
              const int row = r0 + tile * TILE + (int)(es[i] & 63u);
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][row] * v;
            }
          }
        }
        const int ntg = (n_j + tpw - 1) / tpw;
        for (int tg = 0; tg < ntg; ++tg) {
          const uint32_t w =
              vv.codes[((size_t)slab * vv.nblk_cap + (tg >> 2)) * 512 + ((tg & 3) * 16 + (c & 15)) * 8 + (c >> 4)];
          for (int i = 0; i < tpw; ++i) {
            const int t = tg * tpw + i;
            if (t < n_j) {
              const float2 dz = S.vd[(r0 + t) * NG + G];
              const float v = (float)((w >> (i * bits)) & cmask) * dz.x + dz.y;
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][r0 + t] * v;
            }
          }
        }
      }
      for (int k = half; k < nbuf_rows; k += 2) {
        const float v = h2f(Vb[(size_t)(bbase + k) * D + c]);
#pragma unroll
        for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][nrows + k] * v;
      }
#pragma unroll
      for (int hq = 0; hq < GQ; ++hq) S.o_half[half][hq][c] = o[hq];
    }
    // p^T A_V per chunk (down-projection)
    for (int i = tid; i < npc * GQ * 8; i += 256) {
      const int jc = i / (GQ * 8), hq = (i >> 3) % GQ, r = i & 7;
      const int j = jbase + jc, rv = cs.rank[j], n_j = cs.n[j], r0 = S.row0[jc];
      float s = 0.0f;
      if (r < rv) {
        const SegView vv = chunk_view(cs.v0, cs.stride, j, n_j, rv);
        for (int t = 0; t < n_j; ++t) s += S.sc[hq][r0 + t] * h2f(vv.A[((size_t)slab * vv.n_cap + t) * rv + r]);
      }
      S.wv[jc][hq][r] = s;
    }
    // sparse Value term: wave w takes chunks w, w+4, ... into its own plane; lists ordered (c, t)
    if (dm.ppm > 0) {
      for (int jc = wave; jc < npc; jc += 4) {
        const int j = jbase + jc, n_j = cs.n[j];
        const SegView vv = chunk_view(cs.v0, cs.stride, j, n_j, cs.rank[j]);
        for (int tile = 0; tile * TILE < n_j; ++tile) {
          const uint2 oc = S.tabv[jc][tile];
          const uint32_t* lst = vv.sp_pool + (size_t)b * vv.pool_cap + oc.x;
          for (uint32_t e = lane; e < oc.y; e += 64) {
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
              const int row = S.row0[jc] + tile * TILE + (int)((en & 0xFFFFu) >> 7);
#pragma unroll
              for (int hq = 0; hq < GQ; ++hq) a2[hq] += S.sc[hq][row] * v;
            }
#pragma unroll
            for (int hq = 0; hq < GQ; ++hq) S.osp[wave][hq][ch] += a2[hq];
          }
          __builtin_amdgcn_wave_barrier();
        }
      }
    }
    block_lds_sync();
    for (int i = tid; i < GQ * D; i += 256) {
      const int hq = i / D, c = i % D;
      float o = S.o_half[0][hq][c] + S.o_half[1][hq][c];
#pragma unroll
      for (int w = 0; w < 4; ++w) o += S.osp[w][hq][c];
      for (int jc = 0; jc < npc; ++jc) {
        const int j = jbase + jc, rv = cs.rank[j];
        if (rv > 0) {
          const SegView vv = chunk_view(cs.v0, cs.stride, j, cs.n[j], rv);
          for (int r = 0; r < rv; ++r) o += S.wv[jc][hq][r] * h2f(vv.Bf[((size_t)slab * D + c) * rv + r]);
        }
      }
      S.o_run[hq][c] += o;
    }
    j_next += npc;
    buf_done += nbuf_rows;
  }
  block_lds_sync();
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

}  // namespace gear
