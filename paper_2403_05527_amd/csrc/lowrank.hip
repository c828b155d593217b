// SVDSolver_r (Eq. 6, Algorithm 2): batched power iteration on the per-head
// residual R = X - D - S.  The quantization kernels leave Y = X - S (fp16, outliers
// zeroed) in a workspace buffer; every sweep re-derives R = (Y - zero) - code * scale from it
// (Keys: with the stored codes; Values: with the code recomputed by the quantizer's own
// operation sequence).  That is exact (no rounded copy of R) and costs 2 bytes per entry and
// pass, for three more vector instructions per entry than reading a stored remainder; a
// 16-bit copy of R itself flips enough fp16 roundings of the stored factors to fail the
// attention tolerance.
//
//   pi_update  : B <- start matrix or sum of the sweep partials; column scaling
//                between rounds (the span, hence A B^T, is unchanged); QR of B
//                before the last round; after the last round the r x r factor
//                that orthonormalises A, and the final B = R^T orth(A).
//   pi_sweep   : one pass over a slab's residual: a_t = R_t B (per token), partial
//                B' = sum_t R_t^T a_t, and in the last round a_t itself and the
//                Gram matrix sum_t a_t a_t^T.
//   pi_finish  : A = a C  (C = the r x r factor), rounded to fp16.
//   pi_small   : all of the above for a segment of at most 256 tokens, in one block per slab.
#include "gear_internal.h"
#include "gear_launch.h"

namespace gear {

constexpr int PT = 256;  // tokens per sweep block

// Sum over the block (128 or 256 threads; the same value in every thread).
template <typename T>
__device__ __forceinline__ T block_sum(T v, T* red /* 4 */) {
  v = wave_sum_shfl(v);
  block_lds_sync();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  block_lds_sync();
  T s = red[0] + red[1];
  if (blockDim.x > 128) s += red[2] + red[3];
  return s;
}

// grid (B*H), block 128: thread c owns row c of the [128 x R] matrix.
// src_init != nullptr : B <- init (fp32 [slab][128][rank], zero-padded to R)
// else                : B <- sum over `npart` partials ([slab][npart][128*R + R*R])
// do_orth : replace B by the Q factor of its QR (twice-applied modified
//           Gram-Schmidt, fp64; dependent columns become 0)
// final   : also sum the Gram partials, build C with orth(A) = A C, write
//           B_out = B C as fp16 into the arena and C into cmat.
template <int R>
struct UpdateSmem {
  double red[4];
  double G[R][R];
  double C[R][R];
  double cj[R];   // work vector of the one thread that orthonormalises in coefficient space
};
// The body runs in a block of 128 threads (its own kernel) or of 256 (the one-block power
// iteration of short segments, where threads 128.. only take part in the barriers).
template <int R>
__device__ __forceinline__ void pi_update_body(UpdateSmem<R>& sm, int slab, const float* __restrict__ src_init, int rank,
                                               const float* __restrict__ partial, int npart, int do_orth,
                                               int final_round, float* __restrict__ Bcur, float* __restrict__ cmat,
                                               const SegView& sv) {
  double (&G)[R][R] = sm.G;
  double (&C)[R][R] = sm.C;
  double* red = sm.red;
  const int c = threadIdx.x;
  const bool act = c < D;
  double q[R];
#pragma unroll
  for (int r = 0; r < R; ++r) q[r] = 0.0;
  if (act) {
    if (src_init) {
#pragma unroll
      for (int r = 0; r < R; ++r) q[r] = r < rank ? (double)src_init[((size_t)slab * D + c) * rank + r] : 0.0;
    } else {
      const float* p = partial + (size_t)slab * npart * (D * R + R * R);
      for (int i = 0; i < npart; ++i) {
#pragma unroll
        for (int r = 0; r < R; ++r) q[r] += (double)p[(size_t)i * (D * R + R * R) + c * R + r];
      }
    }
  }

  if (final_round) {
    if (c < R * R) {
      const float* p = partial + (size_t)slab * npart * (D * R + R * R) + D * R;
      double s = 0.0;
      for (int i = 0; i < npart; ++i) s += (double)p[(size_t)i * (D * R + R * R) + c];
      G[c / R][c % R] = s;
    }
    block_lds_sync();
    if (c == 0) {
      // Gram-Schmidt in coefficient space: column j of orth(A) is A * C[:, j].
      uint32_t valid = 0;   // bit j: column j is kept
      double* cj = sm.cj;
      for (int j = 0; j < R; ++j) {
        for (int i = 0; i < R; ++i) cj[i] = (i == j) ? 1.0 : 0.0;
        const double before2 = G[j][j];
        bool ok = before2 > 0.0;
        if (ok) {
          for (int pass = 0; pass < 2; ++pass)
            for (int k = 0; k < j; ++k) {
              if (!((valid >> k) & 1u)) continue;
              double dot = 0.0;  // q_k^T v = c_k^T G c_j
              for (int a = 0; a < R; ++a)
                for (int b = 0; b < R; ++b) dot += C[a][k] * G[a][b] * cj[b];
              for (int a = 0; a < R; ++a) cj[a] -= dot * C[a][k];
            }
          double after2 = 0.0;
          for (int a = 0; a < R; ++a)
            for (int b = 0; b < R; ++b) after2 += cj[a] * G[a][b] * cj[b];
          if (!(after2 > 1e-10 * before2)) ok = false;
          else {
            const double inv = 1.0 / sqrt(after2);
            for (int a = 0; a < R; ++a) cj[a] *= inv;
          }
        }
        if (ok) valid |= 1u << j;
        for (int a = 0; a < R; ++a) C[a][j] = ok ? cj[a] : 0.0;
      }
    }
    block_lds_sync();
    double o[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      double s = 0.0;
#pragma unroll
      for (int r = 0; r < R; ++r) s += q[r] * C[r][j];
      o[j] = s;
    }
    if (act)
      for (int j = 0; j < rank; ++j) sv.Bf[((size_t)slab * D + c) * sv.rank + j] = (uint16_t)f2h((float)o[j]);
    if (c < R * R) cmat[(size_t)slab * R * R + c] = (float)C[c / R][c % R];
    return;
  }

  if (do_orth) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const double before2 = block_sum(q[j] * q[j], red);
      if (before2 == 0.0) { q[j] = 0.0; continue; }
      for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
          if (i < j) {
            const double dot = block_sum(q[i] * q[j], red);
            q[j] -= dot * q[i];
          }
        }
      }
      const double after2 = block_sum(q[j] * q[j], red);
      if (!(sqrt(after2) > 1e-12 * sqrt(before2))) q[j] = 0.0;
      else q[j] *= 1.0 / sqrt(after2);
    }
  } else {
    // keep magnitudes in range between rounds
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const double n2 = block_sum(q[j] * q[j], red);
      if (n2 > 0.0) q[j] *= 1.0 / sqrt(n2);
    }
  }
  if (act) {
#pragma unroll
    for (int r = 0; r < R; ++r) Bcur[((size_t)slab * D + c) * R + r] = (float)q[r];
  }
}

template <int R>
__global__ __launch_bounds__(128) void pi_update_kernel(const float* __restrict__ src_init, int rank,
                                                        const float* __restrict__ partial, int npart,
                                                        int do_orth, int final_round,
                                                        float* __restrict__ Bcur, float* __restrict__ cmat,
                                                        SegView sv) {
  __shared__ UpdateSmem<R> sm;
  pi_update_body<R>(sm, blockIdx.x, src_init, rank, partial, npart, do_orth, final_round, Bcur, cmat, sv);
}

// grid (ceil(n/PT), B*H), block 256; thread (r0 = tid/16, oc = tid%16) owns
// channels 8*oc..+7 of rows pt*PT + r0 + 16*k.  Y = X - S in fp16 (what the quantization
// kernel left); the residual R = Y - D-hat = (Y - zero) - code * scale is re-derived per
// entry, so it is exact and costs 2 bytes per entry.  Keys take the code from the stored
// code rows (16 or 32 bits per row piece); Values, whose codes are stored in blocks of
// tokens, recompute it with the quantizer's own operation sequence.  The (zero, 1/scale,
// scale) of the block's groups are prepared once per block in LDS.
// B' += R_t^T a_t runs on the matrix cores: v_mfma_f32_4x4x1 works on 16 blocks of 4 lanes and
// adds, in register i of lane L, a(lane 4*(L/4) + i) * b(lane L).  With a = the lane's
// residual entry e and b = a_t[r = oc % 4], register i of accumulator e holds
// B'[channel 8*(4*(oc/4) + i) + e][r = oc % 4]: 8 instructions per token row instead of 32
// multiply-adds (the sweeps are bound by vector instruction issue, not by HBM).
// LAST: the final round, which also leaves a_t and the Gram matrix (its extra state costs
// one resident block per CU, so the rounds before it are compiled without).
template <bool IS_K, int R>
struct SweepSmem {
  float red[4][D * R];
  float redg[4][R * R];
  // Keys: [2][groups of the block <= 8][128] (zero, scale); Values: [rows][groups of a row <= 4] (zero, 1/scale, scale, -)
  __attribute__((aligned(16))) float prm[IS_K ? 2 * (PT / 32) * D : PT * 4 * 4];
};
// One block's share of a sweep: rows [pt * PT, pt * PT + PT) of slab `slab`, 256 threads.
template <bool IS_K, int R, bool LAST>
__device__ __forceinline__ void pi_sweep_body(SweepSmem<IS_K, R>& sm, int slab, int pt, const uint16_t* __restrict__ Y,
                                              const uint32_t* __restrict__ sv_sz, const uint32_t* __restrict__ sv_codes,
                                              int sv_n_cap, int sv_ng_cap, int g, int bits, int n,
                                              const float* __restrict__ Bcur, float* __restrict__ partial, int npart,
                                              float* __restrict__ Atmp) {
  float (&red)[4][D * R] = sm.red;
  float (&redg)[4][R * R] = sm.redg;
  float* prm = sm.prm;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const uint16_t* Xs = Y + (size_t)slab * n * D;
  const int lg = 31 - __clz(g);   // g is a power of two
  constexpr int GSTR = (PT / 32) * D;   // Keys: floats per parameter plane
  const float qmax = (float)((1 << bits) - 1);
  const uint32_t* crow = sv_codes + (size_t)slab * sv_n_cap * (4 * bits);   // Keys: 128 * bits / 32 words per row

  constexpr int UN = 4;  // rows in flight per thread
  // the rows of an iteration, all requested before the first one is used
  // (buffer views of the slab's rows: a row past the end reads as 0)
  const GEAR_BUF_T xbuf = GEAR_BUF_MAKE(Xs, n * (D * 2));
  const GEAR_BUF_T cbuf = GEAR_BUF_MAKE(crow, IS_K ? n * (16 * bits) : 0);
  const int xoff0 = (pt * PT + r0) * (D * 2) + oc * 16;
  const int coff0 = (pt * PT + r0) * (16 * bits) + oc * (bits == 4 ? 4 : 2);
  auto request = [&](int k0, uint4 (&xv)[UN], uint32_t (&cw)[UN]) {
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      xv[u] = GEAR_BUF_LOAD16_NT(xbuf, xoff0 + 16 * (k0 + u) * (D * 2));
      cw[u] = 0u;
      if (IS_K) {
        const int co = coff0 + 16 * (k0 + u) * (16 * bits);
        cw[u] = bits == 4 ? GEAR_BUF_LOAD4(cbuf, co) : GEAR_BUF_LOAD2(cbuf, co);
      }
    }
  };
  uint4 xv_first[UN];
  uint32_t cw_first[UN];   // Keys: the row piece's 8 codes
  request(0, xv_first, cw_first);   // in flight while the parameters are prepared

  if (IS_K) {
    const int ngb = PT >> lg, grp0 = (pt * PT) >> lg, ng = (n + g - 1) >> lg;
    for (int i = tid; i < ngb * D; i += 256) {
      const int gi = grp0 + (i >> 7);
      GroupQ q;
      q.mn = 0.0f; q.inv = 0.0f; q.delta = 0.0f;
      if (gi < ng) q = load_group(sv_sz[((size_t)slab * sv_ng_cap + gi) * D + (i & 127)]);
      prm[i] = q.mn;
      prm[GSTR + i] = q.delta;
    }
  } else {
    const int ngl = 7 - lg;   // log2 of the groups per row
    for (int i = tid; i < (PT << ngl); i += 256) {
      const int t = pt * PT + (i >> ngl);
      GroupQ q;
      q.mn = 0.0f; q.inv = 0.0f; q.delta = 0.0f;
      if (t < n) q = load_group(sv_sz[(((size_t)slab * sv_n_cap + t) << ngl) + (i & ((1 << ngl) - 1))]);
      *reinterpret_cast<float4*>(&prm[4 * i]) = make_float4(q.mn, q.inv, q.delta, 0.0f);
    }
  }

  float bc[8][R];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int r = 0; r < R; ++r) bc[e][r] = Bcur[((size_t)slab * D + oc * 8 + e) * R + r];

  constexpr int NB = (R + 3) / 4;   // column blocks of four
  floatx4 acc[8][NB];
  float gacc[R];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) acc[e][nb] = floatx4{0.f, 0.f, 0.f, 0.f};
  const bool partial_blk = pt * PT + PT > n;   // block-uniform: only such a block has rows past the end
#pragma unroll
  for (int r = 0; r < R; ++r) gacc[r] = 0.0f;
  block_lds_sync();

#pragma unroll   // no copies of the accumulators at a loop's back edge
  for (int k0 = 0; k0 < PT / 16; k0 += UN) {
    if (pt * PT + 16 * k0 >= n) break;  // block-uniform
    uint4 xv[UN];
    uint32_t cw[UN];
    if (k0 == 0) {
#pragma unroll
      for (int u = 0; u < UN; ++u) { xv[u] = xv_first[u]; cw[u] = cw_first[u]; }
    } else {
      request(k0, xv, cw);
    }
    float pmn[8], pdl[8];   // Keys: parameters of my 8 channels in the current group
    int gi_prev = -1;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int tl = r0 + 16 * (k0 + u), t = pt * PT + tl;
      float vmn = 0.0f, vinv = 0.0f, vdl = 0.0f;   // Values: parameters of my row's channel group
      if (IS_K) {
        const int gi = (16 * (k0 + u)) >> lg;   // group inside the block, block-uniform
        if (gi != gi_prev) {
          const float* pb = &prm[gi * D + oc * 8];
          const float4 a0 = *reinterpret_cast<const float4*>(pb), a1 = *reinterpret_cast<const float4*>(pb + 4);
          const float4 c0 = *reinterpret_cast<const float4*>(pb + GSTR), c1 = *reinterpret_cast<const float4*>(pb + GSTR + 4);
          pmn[0] = a0.x; pmn[1] = a0.y; pmn[2] = a0.z; pmn[3] = a0.w; pmn[4] = a1.x; pmn[5] = a1.y; pmn[6] = a1.z; pmn[7] = a1.w;
          pdl[0] = c0.x; pdl[1] = c0.y; pdl[2] = c0.z; pdl[3] = c0.w; pdl[4] = c1.x; pdl[5] = c1.y; pdl[6] = c1.z; pdl[7] = c1.w;
          gi_prev = gi;
        }
      } else {
        const float4 pv = *reinterpret_cast<const float4*>(&prm[4 * ((tl << (7 - lg)) + ((oc * 8) >> lg))]);
        vmn = pv.x; vinv = pv.y; vdl = pv.z;
      }
      const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
      float cf[8];   // Keys: the stored codes of my 8 channels as floats (one bit-field extract each)
      if (IS_K) {
#pragma unroll
        for (int e = 0; e < 8; ++e) cf[e] = (float)GEAR_UBFE(cw[u], e * bits, bits);
      }
      float res[8];
      float a[R];
#pragma unroll
      for (int r = 0; r < R; ++r) a[r] = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float y = h2f((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
        if (IS_K) {   // the stored code
          res[e] = __builtin_fmaf(-cf[e], pdl[e], y - pmn[e]);
        } else {      // the code the quantizer computed
          res[e] = quant_error(y, vmn, vinv, vdl, qmax);
        }
#pragma unroll
        for (int r = 0; r < R; ++r) a[r] += res[e] * bc[e][r];
      }
      // the 16 lanes of a row hold one token: row sums of a[], delivered where the product
      // B' += R^T a wants them, a_t[4 * nb + oc % 4] in lane oc (0 past R)
      float bsel[NB];
      if constexpr (R == 2) {
        const float u = row16_sum2(a[0], a[1], lane);
        bsel[0] = (oc & 2) ? 0.0f : u;
      } else {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bsel[nb] = row16_sum4(a[4 * nb], a[4 * nb + 1], a[4 * nb + 2], a[4 * nb + 3], lane);
      }
      // Keys: a row past the end has res = -zero-point, not 0; its a_t is dropped instead
      // (Values: the parameters of such rows are 0, so res is)
      if (IS_K && partial_blk && t >= n) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bsel[nb] = 0.0f;
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e][nb] = __builtin_amdgcn_mfma_f32_4x4x1f32(res[e], bsel[nb], acc[e][nb], 0, 0, 0);
      }
      if (LAST) {
        // lane oc < R holds a_t[oc]
        const float mine = (NB > 1 && oc >= 4) ? bsel[NB - 1] : bsel[0];
        if (oc < R && t < n) Atmp[((size_t)slab * n + t) * R + oc] = mine;
        float ar[R];   // the whole a_t in every lane, from the four lanes of the quad
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const float src = bsel[r >> 2];
          ar[r] = (r & 3) == 0 ? dpp_f<0x00>(src) : (r & 3) == 1 ? dpp_f<0x55>(src) : (r & 3) == 2 ? dpp_f<0xAA>(src) : dpp_f<0xFF>(src);
        }
        if (oc < R) {
#pragma unroll
          for (int r = 0; r < R; ++r) gacc[r] += mine * ar[r];
        }
      }
    }
  }

  // reduce over the 16 row-threads that share a channel octet
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float v = acc[e][nb][i];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        acc[e][nb][i] = v;
      }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float v = gacc[r];
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    gacc[r] = v;
  }
  if (lane < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int r = 4 * nb + (oc & 3);
          if (r < R) red[wave][(8 * (4 * (oc >> 2) + i) + e) * R + r] = acc[e][nb][i];
        }
    if (oc < R) {
#pragma unroll
      for (int r = 0; r < R; ++r) redg[wave][oc * R + r] = gacc[r];
    }
  }
  block_lds_sync();
  float* out = partial + ((size_t)slab * npart + pt) * (D * R + R * R);
  for (int i = tid; i < D * R; i += 256) out[i] = red[0][i] + red[1][i] + red[2][i] + red[3][i];
  if (tid < R * R) out[D * R + tid] = LAST ? (redg[0][tid] + redg[1][tid] + redg[2][tid] + redg[3][tid]) : 0.0f;
}

template <bool IS_K, int R, bool LAST>
__global__ __launch_bounds__(256, (R <= 2 ? 4 : R <= 4 ? 3 : 2)) void pi_sweep_kernel(const uint16_t* __restrict__ Y, SegView sv, int g,
                                                       int bits, int n, const float* __restrict__ Bcur,
                                                       float* __restrict__ partial, int npart,
                                                       float* __restrict__ Atmp) {
  __shared__ SweepSmem<IS_K, R> sm;
  pi_sweep_body<IS_K, R, LAST>(sm, blockIdx.y, blockIdx.x, Y, sv.sz, sv.codes, sv.n_cap, sv.ng_cap, g, bits, n, Bcur, partial,
                               npart, Atmp);
}

// A = a C for tokens [256 * pt, 256 * pt + 256) of one slab, one token per thread.  Cs: LDS, R * R floats.
template <int R>
__device__ __forceinline__ void pi_finish_body(float* Cs, int slab, int pt, const float* __restrict__ Atmp,
                                               const float* __restrict__ cmat, const SegView& sv, int n) {
  float* C = Cs;
  if (threadIdx.x < R * R) C[threadIdx.x] = cmat[(size_t)slab * R * R + threadIdx.x];
  block_lds_sync();
  const int t = pt * 256 + threadIdx.x;
  if (t >= n) return;
  float a[R];
#pragma unroll
  for (int r = 0; r < R; ++r) a[r] = Atmp[((size_t)slab * n + t) * R + r];
  for (int j = 0; j < sv.rank; ++j) {
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) s += a[r] * C[r * R + j];
    sv.A[((size_t)slab * sv.n_cap + t) * sv.rank + j] = (uint16_t)f2h(s);
  }
}

// grid (ceil(n/256), B*H), block 256.
template <int R>
__global__ __launch_bounds__(256) void pi_finish_kernel(const float* __restrict__ Atmp,
                                                        const float* __restrict__ cmat, SegView sv, int n) {
  __shared__ float C[R * R];
  pi_finish_body<R>(C, blockIdx.y, blockIdx.x, Atmp, cmat, sv, n);
}

// The whole power iteration of a short segment (n <= PT: a flushed buffer) in one block per
// slab: the same steps as the separate kernels, in the same order and on the same workspace
// arrays, with block barriers where the kernel boundaries were (a slab's steps only depend
// on that slab).  Saves 7 launches of a few microseconds each per tensor.
// grid (B*H), block 256.
template <bool IS_K, int R>
__global__ __launch_bounds__(256, 1) void pi_small_kernel(const uint16_t* __restrict__ Y, SegView sv, int g, int bits,
                                                          int n, int iters, const float* __restrict__ init_B,
                                                          float* __restrict__ Bcur, float* __restrict__ partial,
                                                          float* __restrict__ Atmp, float* __restrict__ cmat) {
  __shared__ UpdateSmem<R> um;
  __shared__ SweepSmem<IS_K, R> ss;
  __shared__ float Cs[R * R];
  const int slab = blockIdx.x;
  pi_update_body<R>(um, slab, init_B, sv.rank, nullptr, 0, iters == 1 ? 1 : 0, 0, Bcur, cmat, sv);
  __syncthreads();   // also orders the block's global writes before its reads
#pragma unroll 1
  for (int l = 0; l < iters; ++l) {
    const int last = (l == iters - 1);
    // the rounds read the same Y, codes and scales: an offset the compiler cannot see through
    // keeps it from hoisting those loads out of the loop (and holding them in registers)
    int off = 0;
    GEAR_PIN_VGPR(off);
    if (last)
      pi_sweep_body<IS_K, R, true>(ss, slab, 0, Y + off, sv.sz + off, sv.codes + off, sv.n_cap, sv.ng_cap, g, bits, n, Bcur,
                                   partial, 1, Atmp);
    else
      pi_sweep_body<IS_K, R, false>(ss, slab, 0, Y + off, sv.sz + off, sv.codes + off, sv.n_cap, sv.ng_cap, g, bits, n, Bcur,
                                    partial, 1, Atmp);
    __syncthreads();
    pi_update_body<R>(um, slab, nullptr, sv.rank, partial, 1, (l == iters - 2) ? 1 : 0, last, Bcur, cmat, sv);
    __syncthreads();
  }
  pi_finish_body<R>(Cs, slab, 0, Atmp, cmat, sv, n);
}

// ------------------------------------------------------------------ host side
template <int R>
static hipError_t run_pi(bool is_k, const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int iters,
                         const float* init_B, float* Bcur, float* partial, float* Atmp, float* cmat,
                         hipStream_t st) {
  const int slabs = dm.B * dm.H;
  const int npart = (n + PT - 1) / PT;
  if (npart == 1) {   // a short segment: everything in one block per slab
    if (is_k)
      hipLaunchKernelGGL((pi_small_kernel<true, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, iters, init_B, Bcur, partial, Atmp, cmat);
    else
      hipLaunchKernelGGL((pi_small_kernel<false, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, iters, init_B, Bcur, partial, Atmp, cmat);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(pi_update_kernel<R>, dim3(slabs), dim3(128), 0, st, init_B, sv.rank, (const float*)nullptr,
                     0, iters == 1 ? 1 : 0, 0, Bcur, cmat, sv);
  for (int l = 0; l < iters; ++l) {
    const int last = (l == iters - 1);
    const dim3 grid(npart, slabs);
    if (is_k && last)
      hipLaunchKernelGGL((pi_sweep_kernel<true, R, true>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, (const float*)Bcur, partial, npart, Atmp);
    else if (is_k)
      hipLaunchKernelGGL((pi_sweep_kernel<true, R, false>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, (const float*)Bcur, partial, npart, Atmp);
    else if (last)
      hipLaunchKernelGGL((pi_sweep_kernel<false, R, true>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, (const float*)Bcur, partial, npart, Atmp);
    else
      hipLaunchKernelGGL((pi_sweep_kernel<false, R, false>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, (const float*)Bcur, partial, npart, Atmp);
    hipLaunchKernelGGL(pi_update_kernel<R>, dim3(slabs), dim3(128), 0, st, (const float*)nullptr, sv.rank,
                       (const float*)partial, npart, (l == iters - 2) ? 1 : 0, last, Bcur, cmat, sv);
  }
  hipLaunchKernelGGL(pi_finish_kernel<R>, dim3((n + 255) / 256, slabs), dim3(256), 0, st, (const float*)Atmp,
                     (const float*)cmat, sv, n);
  return hipGetLastError();
}

int pi_padded_rank(int rank) { return rank <= 2 ? 2 : rank <= 4 ? 4 : 8; }

hipError_t launch_power_iteration(bool is_k, const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int iters,
                                  const float* init_B, float* Bcur, float* partial, float* Atmp, float* cmat,
                                  hipStream_t st) {
  switch (pi_padded_rank(sv.rank)) {
    case 2: return run_pi<2>(is_k, Yf, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
    case 4: return run_pi<4>(is_k, Yf, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
    default: return run_pi<8>(is_k, Yf, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
  }
}

}  // namespace gear
