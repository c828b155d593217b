// Attention over the fp16 streaming buffer (the rows not yet compressed, Algorithm 1)
// for one (b, h_kv): a plain-ALU block, one thread per buffer row for the scores, one
// thread per (channel, row parity) for the Value side.  Appended chunk segments do not
// come here: they go through the matrix-core block like the prefill.
#pragma once
#include "gear_internal.h"
#include "gear_launch.h"

namespace gear {

constexpr int TAIL_ROWS = 256;   // >= the largest buffer (n_buf_cap <= 255)

template <int GQ>
struct TailSmem {
  float q[GQ][D];
  float sc[GQ][TAIL_ROWS];
  float o_half[2][GQ][D];
  float red[GQ][4];
  float stat[GQ][2];   // m, l
};

// View of chunk j: the chunk regions lie `stride` bytes apart and share one layout.
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

// Kb, Vb: the slab's buffer rows [n_buf][128] fp16.  Writes the record (m, l, o[128]) of each of
// the GQ query columns; m = -inf, l = 0 when a column sees no buffer row.  A column is one query
// row of one query head: column hq holds query row hq % q_len, and with `causal` that query sees
// the buffer rows 0 .. n_buf - q_len + hq % q_len only (the q_len newest tokens are the buffer's
// last q_len rows); q_len = 1: the single-query read, every column sees all n_buf rows.
template <int GQ>
__device__ __forceinline__ void buffer_block(TailSmem<GQ>& S, const uint16_t* __restrict__ qg, const uint16_t* __restrict__ Kb,
                             const uint16_t* __restrict__ Vb, int n_buf, int q_len, int causal,
                             float* __restrict__ rec_base, int rec_stride) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float scale = 0.08838834764831845f;  // 1/sqrt(128)
  // Scores: thread (row16 = tid / 16, piece = tid % 16) takes the 16-byte piece (8 channels) of rows
  // row16, row16 + 16, ...; the 16 lanes of a row add their partial dot products.  The loads that do not
  // depend on the scores are requested before anything waits: q, the pieces of the first two rows, and
  // the first eight Value rows of the thread's (channel, parity) on the Value side.
  const int row16 = tid >> 4, piece = tid & 15;
  auto load_piece = [&](int row) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < n_buf) v = reinterpret_cast<const uint4*>(Kb + (size_t)row * D)[piece];
    return v;
  };
  const uint4 kp0 = load_piece(row16), kp1 = load_piece(row16 + 16);
  const int vc = tid & 127, vhalf = tid >> 7;
  uint32_t vr0[4];   // two fp16 values per word
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int k = vhalf + 4 * u;
    uint32_t a = 0, b = 0;
    if (k < n_buf) a = Vb[(size_t)k * D + vc];
    if (k + 2 < n_buf) b = Vb[(size_t)(k + 2) * D + vc];
    vr0[u] = a | (b << 16);
  }
  for (int i = tid; i < GQ * D; i += 256) S.q[i / D][i % D] = h2f(qg[i]);
  block_lds_sync();
  auto row_scores = [&](const uint4& kv, int row) {   // raw scores of `row` into S.sc
    const uint32_t w[4] = {kv.x, kv.y, kv.z, kv.w};
    float kf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) kf[e] = h2f((w[e >> 1] >> ((e & 1) * 16)) & 0xFFFFu);
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) {
      const float4 a = *reinterpret_cast<const float4*>(&S.q[hq][piece * 8]);   // q of the thread's 8 channels
      const float4 b = *reinterpret_cast<const float4*>(&S.q[hq][piece * 8 + 4]);
      float p = a.x * kf[0] + a.y * kf[1] + a.z * kf[2] + a.w * kf[3] + b.x * kf[4] + b.y * kf[5] + b.z * kf[6] + b.w * kf[7];
      p = row16_sum(p);
      if (piece == 0 && row < n_buf) S.sc[hq][row] = p;
    }
  };
  row_scores(kp0, row16);
  row_scores(kp1, row16 + 16);
  for (int r0 = 32; r0 < n_buf; r0 += 16) row_scores(load_piece(r0 + row16), r0 + row16);
  block_lds_sync();
  float s[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) s[hq] = tid < n_buf ? S.sc[hq][tid] : 0.0f;
  // ---- softmax over the buffer rows
  float p[GQ];
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    const int seen = causal ? n_buf - q_len + 1 + (hq & (q_len - 1)) : n_buf;   // q_len is a power of two
    s[hq] = tid < seen ? s[hq] * scale : -INFINITY;
    const float mx = wave_max(s[hq]);
    if (lane == 0) S.red[hq][wave] = mx;
  }
  block_lds_sync();
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    const float m = fmaxf(fmaxf(S.red[hq][0], S.red[hq][1]), fmaxf(S.red[hq][2], S.red[hq][3]));
    p[hq] = s[hq] > -INFINITY ? __expf(s[hq] - m) : 0.0f;
    S.sc[hq][tid] = p[hq];
    if (tid == 0) S.stat[hq][0] = m;
  }
  block_lds_sync();
#pragma unroll
  for (int hq = 0; hq < GQ; ++hq) {
    const float sum = wave_sum(p[hq]);
    if (lane == 0) S.red[hq][wave] = sum;
  }
  // ---- Value side: thread (channel c, parity) walks rows parity, parity + 2, ...; 8 rows in flight
  // (the first eight were requested at the start)
  {
    const int c = vc, half = vhalf;
    float o[GQ];
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) o[hq] = 0.0f;
    for (int k0 = half; k0 < n_buf; k0 += 16) {
      uint16_t vr[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + 2 * u;
        vr[u] = 0;
        if (k0 == half) vr[u] = (uint16_t)(vr0[u >> 1] >> ((u & 1) * 16));
        else if (k < n_buf) vr[u] = Vb[(size_t)k * D + c];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int k = k0 + 2 * u;
        if (k < n_buf) {
          const float v = h2f(vr[u]);
#pragma unroll
          for (int hq = 0; hq < GQ; ++hq) o[hq] += S.sc[hq][k] * v;
        }
      }
    }
#pragma unroll
    for (int hq = 0; hq < GQ; ++hq) S.o_half[half][hq][c] = o[hq];
  }
  block_lds_sync();
  for (int i = tid; i < GQ * D; i += 256) {
    const int hq = i / D, c = i % D;
    float* rec = rec_base + (size_t)hq * rec_stride;
    rec[2 + c] = S.o_half[0][hq][c] + S.o_half[1][hq][c];
    if (c == 0) {
      rec[0] = S.stat[hq][0];
      rec[1] = S.red[hq][0] + S.red[hq][1] + S.red[hq][2] + S.red[hq][3];
    }
  }
}

}  // namespace gear
