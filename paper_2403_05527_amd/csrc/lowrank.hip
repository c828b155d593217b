// SVDSolver_r (Eq. 6, Algorithm 2): batched power iteration on the per-head
// residual R = X - D - S.  The quantization kernels leave Y = X - S (fp16, outliers
// zeroed) in a workspace buffer; every sweep re-derives R = (Y - zero) - code * scale from it
// (Keys: with the stored codes; Values: with the code recomputed by the quantizer's own
// operation sequence).  That is exact (no rounded copy of R) and costs 2 bytes per entry and
// pass, for three more vector instructions per entry than reading a stored remainder; a
// 16-bit copy of R itself flips enough fp16 roundings of the stored factors to fail the
// attention tolerance.
//
//   pi_gram    : G = R^T R (128 x 128 per slab) in one pass over the residual, on the
//                matrix cores.  Every round of Algorithm 2 before the last maps
//                B -> R^T (R B) = G B, so those rounds need no pass over R of their
//                own: they become 128 x 128 x r products on G.
//   pi_solve   : B <- G^(L-1) B0 (columns rescaled between the products: the span,
//                hence A B^T, is unchanged), then the QR of B that opens the last round.
//                With L > 1 the last round comes out of G as well: for A = R Q (Q = that
//                orthonormal B), A^T A = Q^T G Q gives the r x r factor C with orth(A) = A C,
//                and the final B = R^T orth(A) = G Q C; the kernel writes B (fp16) and W = Q C.
//   pi_project : A = R W per token, rounded to fp16: the one pass over R of the last round.
//   (L = 1 has no Gram pass; its single round runs as sweep + update + finish below.)
//   pi_update  : B <- start matrix or sum of the sweep partials; column scaling
//                between rounds (the span, hence A B^T, is unchanged); QR of B
//                before the last round; after the last round the r x r factor
//                that orthonormalises A, and the final B = R^T orth(A).
//   pi_sweep   : one pass over a slab's residual: a_t = R_t B (per token), partial
//                B' = sum_t R_t^T a_t, and in the last round a_t itself and the
//                Gram matrix sum_t a_t a_t^T.
//   pi_finish  : A = a C  (C = the r x r factor), rounded to fp16.
//   pi_small   : all of the above for a segment of at most 256 tokens, in one block per slab.
//   pi_tiny    : a segment of at most 64 tokens (a flushed buffer): one block per slab with the residual in LDS.
#include <atomic>
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

// Sum of a double over the 64 lanes, in every lane: lane exchanges inside rows of 16 (one
// data-parallel-primitive move per 32-bit half), then the four row sums through scalar reads.
template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = dpp_u<CTRL>((uint32_t)b), hi = dpp_u<CTRL>((uint32_t)(b >> 32));
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double lane_bcast_d(double v, int lane) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), lane);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double wave_sum_d(double v) {
  v += dpp_d<DPP_XOR1>(v);
  v += dpp_d<DPP_XOR2>(v);
  v += dpp_d<DPP_HALF_MIRROR>(v);
  v += dpp_d<DPP_MIRROR>(v);
  return (lane_bcast_d(v, 0) + lane_bcast_d(v, 16)) + (lane_bcast_d(v, 32) + lane_bcast_d(v, 48));
}
// Gram-Schmidt (applied twice) in coefficient space: given the r x r Gram matrix G = A^T A of the columns of some A, finds C
// with orth(A) = A C (column j of orth(A) is A * C[:, j]; dependent columns get C[:, j] = 0).  Called by the
// 64 threads c = 0..63 of one wave; lane a * R + b carries the (a, b) term of every quadratic form x^T G y, a
// sum over the wave finishes it.  G, C, cj: LDS.
template <int R>
__device__ __forceinline__ void coeff_orth(double (&G)[R][R], double (&C)[R][R], double* cj, int c) {
  const int a = c / R, b = c % R;
  const bool in = c < R * R;
  const double Gab = in ? G[a][b] : 0.0;
  uint32_t valid = 0;   // bit j: column j is kept
  for (int j = 0; j < R; ++j) {
    if (c < R) cj[c] = (c == j) ? 1.0 : 0.0;
    wave_lds_sync();
    const double before2 = G[j][j];
    bool ok = before2 > 0.0;
    if (ok) {
      // two passes; the projections of a pass are taken together from the same vector (their reductions
      // are independent of each other and overlap), then removed together
      for (int pass = 0; pass < 2; ++pass) {
        double dot[R];
#pragma unroll
        for (int k = 0; k < R; ++k) {
          dot[k] = 0.0;
          if (k < j && ((valid >> k) & 1u)) dot[k] = wave_sum_d(in ? C[a][k] * Gab * cj[b] : 0.0);   // q_k^T v = c_k^T G c_j
        }
        wave_lds_sync();
        if (c < R) {
          double v = cj[c];
#pragma unroll
          for (int k = 0; k < R; ++k)
            if (k < j) v -= dot[k] * C[c][k];
          cj[c] = v;
        }
        wave_lds_sync();
      }
      const double after2 = wave_sum_d(in ? cj[a] * Gab * cj[b] : 0.0);
      wave_lds_sync();
      // (the Gram matrix is a sum of fp32 products: what is left of a dependent column is
      // rounding noise of relative size ~1e-7 in after2, so the cut sits above that)
      if (!(after2 > 1e-6 * before2)) ok = false;
      else {
        const double inv = 1.0 / sqrt(after2);
        if (c < R) cj[c] *= inv;
        wave_lds_sync();
      }
    }
    if (ok) valid |= 1u << j;
    if (c < R) C[c][j] = ok ? cj[c] : 0.0;
    wave_lds_sync();
  }
}

// grid (B*H), block 256: thread c < 128 owns row c of the [128 x R] matrix.
// from_start          : B <- the start matrix (zero-padded to R)
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
// The body runs in a block of 256 threads: threads 128.. sum the Gram partials of the final round
// and otherwise only take part in the barriers.
template <int R>
__device__ __forceinline__ void pi_update_body(UpdateSmem<R>& sm, int slab, bool from_start, const StartB& sb, int rank,
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
    if (from_start) {
#pragma unroll
      for (int r = 0; r < R; ++r) q[r] = r < rank ? (double)start_b(sb, slab, c, rank, r) : 0.0;
    } else {
      const float* p = partial + (size_t)slab * npart * (D * R + R * R);
      int i = 0;
      // long segments (many partials): the loads of eight partials are requested before the first is added
      // (written as a load loop of its own: an add right after its load makes the compiler wait for every load)
      if (npart > 16) {
        for (; i + 8 <= npart; i += 8) {
          float t[8][R];
#pragma unroll
          for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r) t[u][r] = __builtin_nontemporal_load(&p[(size_t)(i + u) * (D * R + R * R) + c * R + r]);
#pragma unroll
          for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int r = 0; r < R; ++r) q[r] += (double)t[u][r];
        }
      }
      for (; i < npart; ++i) {
#pragma unroll
        for (int r = 0; r < R; ++r) q[r] += (double)p[(size_t)i * (D * R + R * R) + c * R + r];
      }
    }
  }

  if (final_round) {
    if (c >= D && c < D + R * R) {   // threads 128..: the r x r Gram partials, while threads 0..127 sum theirs
      const int gi = c - D;
      const float* p = partial + (size_t)slab * npart * (D * R + R * R) + D * R + gi;
      double s = 0.0;
      int i = 0;
      for (; i + 8 <= npart; i += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = __builtin_nontemporal_load(&p[(size_t)(i + u) * (D * R + R * R)]);
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (double)t[u];
      }
      for (; i < npart; ++i) s += (double)p[(size_t)i * (D * R + R * R)];
      G[gi / R][gi % R] = s;
    }
    block_lds_sync();
    if (c < 64) coeff_orth<R>(G, C, sm.cj, c);
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
__global__ __launch_bounds__(256) void pi_update_kernel(int from_start, StartB sb, int rank,
                                                        const float* __restrict__ partial, int npart,
                                                        int do_orth, int final_round,
                                                        float* __restrict__ Bcur, float* __restrict__ cmat,
                                                        SegView sv) {
  __shared__ UpdateSmem<R> sm;
  pi_update_body<R>(sm, blockIdx.x, from_start != 0, sb, rank, partial, npart, do_orth, final_round, Bcur, cmat, sv);
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
// PROJECT: only A = R B is wanted, and it is the final A (B holds the projection matrix of the last round):
// rows go to the arena as fp16, nothing is accumulated.
template <bool IS_K, int R, bool LAST, bool PROJECT = false>
__device__ __forceinline__ void pi_sweep_body(SweepSmem<IS_K, R>& sm, int slab, int pt, const uint16_t* __restrict__ Y,
                                              const uint32_t* __restrict__ sv_sz, const uint32_t* __restrict__ sv_codes,
                                              int sv_n_cap, int sv_ng_cap, int g, int bits, int n, int t_lr,
                                              const float* __restrict__ Bcur, float* __restrict__ partial, int npart,
                                              float* __restrict__ Atmp, uint16_t* __restrict__ A_out = nullptr, int rank = 0) {
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
    const int ngb = (PT >> lg) > 0 ? (PT >> lg) : 1, grp0 = (pt * PT) >> lg, ng = (n + g - 1) >> lg;
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
      // rows before t_lr take no part in the low-rank term (error reduction on the most recent tokens only)
      if ((IS_K && partial_blk && t >= n) || t < t_lr) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bsel[nb] = 0.0f;
      }
      if constexpr (PROJECT) {
        // lane oc < R holds a_t[oc]
        const float mine = (NB > 1 && oc >= 4) ? bsel[NB - 1] : bsel[0];
        if (oc < rank && t < n) A_out[((size_t)slab * sv_n_cap + t) * rank + oc] = (uint16_t)f2h(mine);
        continue;
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

  if constexpr (PROJECT) return;
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
                                                       int bits, int n, int t_lr, const float* __restrict__ Bcur,
                                                       float* __restrict__ partial, int npart,
                                                       float* __restrict__ Atmp) {
  __shared__ SweepSmem<IS_K, R> sm;
  pi_sweep_body<IS_K, R, LAST>(sm, blockIdx.y, blockIdx.x, Y, sv.sz, sv.codes, sv.n_cap, sv.ng_cap, g, bits, n, t_lr, Bcur, partial,
                               npart, Atmp);
}

// The pass of the last round when the Gram matrix exists: A = R W with the projection matrix W that
// pi_solve_kernel left in Bcur, written to the arena as fp16.  grid (ceil(n / 256), B*H), block 256.
template <bool IS_K, int R>
__global__ __launch_bounds__(256, (R <= 4 ? 4 : 3)) void pi_project_kernel(const uint16_t* __restrict__ Y, SegView sv, int g, int bits,
                                                                         int n, int t_lr, const float* __restrict__ Bcur) {
  __shared__ SweepSmem<IS_K, R> sm;
  pi_sweep_body<IS_K, R, false, true>(sm, blockIdx.y, blockIdx.x, Y, sv.sz, sv.codes, sv.n_cap, sv.ng_cap, g, bits, n, t_lr, Bcur,
                                      nullptr, 0, nullptr, sv.A, sv.rank);
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
                                                          int n, int t_lr, int iters, StartB sb,
                                                          float* __restrict__ Bcur, float* __restrict__ partial,
                                                          float* __restrict__ Atmp, float* __restrict__ cmat) {
  __shared__ UpdateSmem<R> um;
  __shared__ SweepSmem<IS_K, R> ss;
  __shared__ float Cs[R * R];
  const int slab = blockIdx.x;
  pi_update_body<R>(um, slab, true, sb, sv.rank, nullptr, 0, iters == 1 ? 1 : 0, 0, Bcur, cmat, sv);
  __syncthreads();   // also orders the block's global writes before its reads
#pragma unroll 1
  for (int l = 0; l < iters; ++l) {
    const int last = (l == iters - 1);
    // the rounds read the same Y, codes and scales: an offset the compiler cannot see through
    // keeps it from hoisting those loads out of the loop (and holding them in registers)
    int off = 0;
    GEAR_PIN_VGPR(off);
    if (last)
      pi_sweep_body<IS_K, R, true>(ss, slab, 0, Y + off, sv.sz + off, sv.codes + off, sv.n_cap, sv.ng_cap, g, bits, n, t_lr, Bcur,
                                   partial, 1, Atmp);
    else
      pi_sweep_body<IS_K, R, false>(ss, slab, 0, Y + off, sv.sz + off, sv.codes + off, sv.n_cap, sv.ng_cap, g, bits, n, t_lr, Bcur,
                                    partial, 1, Atmp);
    __syncthreads();
    pi_update_body<R>(um, slab, false, sb, sv.rank, partial, 1, (l == iters - 2) ? 1 : 0, last, Bcur, cmat, sv);
    __syncthreads();
  }
  pi_finish_body<R>(Cs, slab, 0, Atmp, cmat, sv, n);
}

// ------------------------------------------------------------------ Gram matrix of the residual
// Rounds 1 .. L-1 of Algorithm 2 compute A = R B, B = R^T A without any orthonormalisation in
// between, i.e. B <- (R^T R) B.  G = R^T R is formed once, in one pass over the slab, as a dense
// contraction over the tokens on v_mfma_f32_16x16x32_f16; the rounds themselves then cost
// 128 x 128 x r multiply-adds per slab (pi_solve_kernel).  A residual entry enters the
// contraction as two fp16 numbers, its leading part and what that leaves (22 bits together), and
// a product as three MFMA terms; accumulation is fp32.  (The leading parts alone are not enough:
// without orthonormalisation between the rounds the weaker directions of G^(L-1) B0 are small
// differences of large numbers, and a relative error of 2^-11 in G is amplified by the square
// of the ratio of its leading eigenvalues.)  G only chooses the subspace that the last round
// projects on: that round (pi_sweep_kernel<.., LAST>) still reads the residual itself, so
// A = orth(R B) and B = R^T A are computed from R.
//
// grid (ceil(n / strip), B*H), block 256.  A block walks its strip of tokens in steps of 128;
// thread (r0 = tid/16, oc = tid%16) takes channels 8*oc..+7 of rows base + r0 + 16*k, k = 0..7.
// The 16 lanes that share r0 hold the same 8 tokens: as an MFMA operand, register j of
// "channel e" holds rows (2j, 2j+1) of channel 8*oc + e, so operand e is the 16 channels
// {8*oc + e} x 32 tokens of the wave and acc(e, e') += op_e^T op_e' is one 16 x 16 tile of G:
// lane l, register i <-> G[8*(4*(l/16)+i) + e][8*(l%16) + e'].  Only the 36 tiles e <= e' are
// computed (G is symmetric).  The four waves' tiles are summed through LDS and written as one
// partial per strip: [slab][strip][36][4][64] floats.
constexpr int GRAM_TILES = 36;
constexpr int GRAM_FLOATS = GRAM_TILES * 256;

typedef _Float16 gram_h2 __attribute__((ext_vector_type(2)));
typedef _Float16 gram_h8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ uint32_t pack_h2(float a, float b) {   // two roundings to nearest even, one instruction
  gram_h2 h = {(_Float16)a, (_Float16)b};
  return __builtin_bit_cast(uint32_t, h);
}

// The loads of one step of the Gram pass (128 tokens, 8 rows per thread), requested together.
template <bool IS_K, int NGS>
struct GramLoads {
  uint4 xv[8];
  uint32_t cw[8];      // Keys: the row piece's 8 codes
  uint32_t pv[8];      // Values: (scale, zero) of my row's channel group
  uint4 pz[NGS][2];    // Keys: (scale, zero) of my 8 channels in the step's groups
};

template <bool IS_K, int LG>   // LG: log2 of the Key group size (Values take the group size at run time)
__global__ __launch_bounds__(256, 2) void pi_gram_kernel(const uint16_t* __restrict__ Y, SegView sv, int g, int bits, int n,
                                                         int t_lr, int strip, float* __restrict__ gram_partial) {
  __shared__ float red[GRAM_FLOATS];
  const int slab = blockIdx.y, sidx = blockIdx.x, nstrips = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const int t_begin = sidx * strip;
  const int t_end = t_begin + strip < n ? t_begin + strip : n;
  const float qmax = (float)((1 << bits) - 1);
  const int lgv = 31 - __clz(g), ngl = 7 - lgv;   // Values: log2 of the group size / of the groups per row
  const GEAR_BUF_T xbuf = GEAR_BUF_MAKE(Y + (size_t)slab * n * D, n * (D * 2));
  const GEAR_BUF_T cbuf = GEAR_BUF_MAKE(sv.codes + (size_t)slab * sv.n_cap * (4 * bits), IS_K ? n * (16 * bits) : 0);
  // (scale, zero) words: Keys [group][128] of this slab, Values [row][groups of a row]
  const GEAR_BUF_T pbuf = IS_K ? GEAR_BUF_MAKE(sv.sz + (size_t)slab * sv.ng_cap * D, ((n + g - 1) >> LG) * (D * 4))
                               : GEAR_BUF_MAKE(sv.sz + (((size_t)slab * sv.n_cap) << ngl), (n << ngl) * 4);
  constexpr int GT = 128;                          // tokens per step (32 per wave)
  constexpr int NGS = (IS_K && (GT >> LG) > 0) ? (GT >> LG) : 1;   // Key groups per step
  typedef GramLoads<IS_K, NGS> Loads;

  floatx4 acc[GRAM_TILES];
#pragma unroll
  for (int i = 0; i < GRAM_TILES; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

#pragma unroll 1
  for (int base = t_begin; base < t_end; base += GT) {
    // every load of the step is requested before the first one is used
    Loads L;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int t = base + r0 + 16 * k;
      L.xv[k] = GEAR_BUF_LOAD16_NT(xbuf, t * (D * 2) + oc * 16);   // rows past the end read as 0
      L.cw[k] = 0u;
      L.pv[k] = 0u;
      if (IS_K) {
        const int co = t * (16 * bits) + oc * (bits == 4 ? 4 : 2);
        L.cw[k] = bits == 4 ? GEAR_BUF_LOAD4(cbuf, co) : GEAR_BUF_LOAD2(cbuf, co);
      } else {
        L.pv[k] = GEAR_BUF_LOAD4(pbuf, ((t << ngl) + ((oc * 8) >> lgv)) * 4);
      }
    }
    if (IS_K) {
#pragma unroll
      for (int j = 0; j < NGS; ++j) {
        const int off = (((base >> LG) + j) * D + oc * 8) * 4;
        L.pz[j][0] = GEAR_BUF_LOAD16(pbuf, off);
        L.pz[j][1] = GEAR_BUF_LOAD16(pbuf, off + 16);
      }
    }
    // residuals of the step as fp16 operands: leading part, and what it leaves (22 bits together)
    const bool ragged = base + GT > n;   // block-uniform: only such a step has rows past the end
    uint32_t oph[8][4], opl[8][4];
    float pmn[8], pdl[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { pmn[e] = 0.0f; pdl[e] = 0.0f; }
    float ra[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t w[4] = {L.xv[k].x, L.xv[k].y, L.xv[k].z, L.xv[k].w};
      float res[8];
      if (IS_K) {
        if ((16 * k) % (1 << (LG < 8 ? LG : 8)) == 0) {   // first rows of a group: its parameters
          const int j = (16 * k) >> LG;
          const uint32_t z[8] = {L.pz[j][0].x, L.pz[j][0].y, L.pz[j][0].z, L.pz[j][0].w,
                                 L.pz[j][1].x, L.pz[j][1].y, L.pz[j][1].z, L.pz[j][1].w};
#pragma unroll
          for (int e = 0; e < 8; ++e) { pdl[e] = h2f(z[e] & 0xFFFFu); pmn[e] = h2f(z[e] >> 16); }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = h2f((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
          res[e] = __builtin_fmaf(-(float)GEAR_UBFE(L.cw[k], e * bits, bits), pdl[e], y - pmn[e]);
        }
      } else {
        const GroupQ q = load_group(L.pv[k]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = h2f((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
          res[e] = quant_error(y, q.mn, q.inv, q.delta, qmax);
        }
      }
      // Keys: a row past the end has res = -zero-point, not 0 (Values: the parameters of such rows are 0)
      // (rows before t_lr take no part in the low-rank term)
      if ((IS_K && ragged && base + r0 + 16 * k >= n) || base + r0 + 16 * k < t_lr) {
#pragma unroll
        for (int e = 0; e < 8; ++e) res[e] = 0.0f;
      }
      if ((k & 1) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) ra[e] = res[e];
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t hi = pack_h2(ra[e], res[e]);
          oph[e][k >> 1] = hi;
          opl[e][k >> 1] = pack_h2(ra[e] - h2f(hi & 0xFFFFu), res[e] - h2f(hi >> 16));
        }
      }
    }
    // the 36 tiles: r r' = hi hi' + hi lo' + lo hi' (the lo lo' term is below fp32 resolution)
    int ti = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const gram_h8 ah = __builtin_bit_cast(gram_h8, make_uint4(oph[e][0], oph[e][1], oph[e][2], oph[e][3]));
      const gram_h8 al = __builtin_bit_cast(gram_h8, make_uint4(opl[e][0], opl[e][1], opl[e][2], opl[e][3]));
#pragma unroll
      for (int f = e; f < 8; ++f) {
        const gram_h8 bh = __builtin_bit_cast(gram_h8, make_uint4(oph[f][0], oph[f][1], oph[f][2], oph[f][3]));
        const gram_h8 bl = __builtin_bit_cast(gram_h8, make_uint4(opl[f][0], opl[f][1], opl[f][2], opl[f][3]));
        acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bh, acc[ti], 0, 0, 0);
        acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, bl, acc[ti], 0, 0, 0);
        acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, bh, acc[ti], 0, 0, 0);
        ++ti;
      }
    }
  }

  // the four waves' tiles, added in wave order (a fixed order: results do not vary from run to run);
  // a few tiles at a time, so that the LDS reads in flight stay few
  float* out = gram_partial + ((size_t)slab * nstrips + sidx) * GRAM_FLOATS;
  if (wave == 0) {
#pragma unroll
    for (int ti = 0; ti < GRAM_TILES; ++ti)
#pragma unroll
      for (int i = 0; i < 4; ++i) red[ti * 256 + i * 64 + lane] = acc[ti][i];
  }
  block_lds_sync();
#pragma unroll 1
  for (int w = 1; w < 3; ++w) {
    if (wave == w) {
#pragma unroll
      for (int ti = 0; ti < GRAM_TILES; ++ti) {
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = red[ti * 256 + i * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) red[ti * 256 + i * 64 + lane] = v[i] + acc[ti][i];
        GEAR_PIN_VGPR(v[0]);   // keeps the tiles' reads from being hoisted above each other's writes en bloc
      }
    }
    block_lds_sync();
  }
  if (wave == 3) {
#pragma unroll
    for (int ti = 0; ti < GRAM_TILES; ++ti) {
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = red[ti * 256 + i * 64 + lane];
#pragma unroll
      for (int i = 0; i < 4; ++i) out[ti * 256 + i * 64 + lane] = v[i] + acc[ti][i];
      GEAR_PIN_VGPR(v[0]);
    }
  }
}

// B <- G^rounds B0, then the Q factor of its QR (the orthonormalisation of B that opens the last
// round of Algorithm 2).  grid (B*H), block 128: thread c owns row c of B.  Dynamic LDS: G as
// [128][129] floats, B as [128][R] doubles.
constexpr int GP = D + 1;
template <int R>
struct SolveSmem {
  float G[D * GP];
  double Bs[D][R];
  float part[D][R];    // the upper half block's share of a product (single precision: with it two blocks fit a CU)
  double red[4 * (R + 1)];
  double GA[R][R];     // the last round: Gram matrix of A = R B, the factor C of its orthonormalisation
  double C[R][R];
  double cj[R];
};
// Sums of N per-thread values over the block (256 threads), all in every thread: one pair of
// barriers for the N sums together.
template <int N>
__device__ __forceinline__ void block_sum_vec(double (&v)[N], double* red /* 4 * N */) {
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = wave_sum_d(v[i]);
  block_lds_sync();
  if ((threadIdx.x & 63) == 0) {
#pragma unroll
    for (int i = 0; i < N; ++i) red[(threadIdx.x >> 6) * N + i] = v[i];
  }
  block_lds_sync();
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = (red[i] + red[N + i]) + (red[2 * N + i] + red[3 * N + i]);
}
// 1 / sqrt(x) for x > 0 in double: the single-precision estimate, refined by two Newton steps
// (no double-precision square root or division, which are long instruction sequences)
__device__ __forceinline__ double rsqrt_d(double x) {
  // scaled into single-precision range by an even power of two taken from the exponent
  const int ex = (int)((__builtin_bit_cast(uint64_t, x) >> 52) & 0x7FF) - 1023;
  const int h = ex >> 1;                                   // x = m * 4^h, m in [1, 4)
  const double m = __builtin_bit_cast(double, __builtin_bit_cast(uint64_t, x) - ((uint64_t)(2 * h) << 52));
  double y = (double)__builtin_amdgcn_rsqf((float)m);
  y = y * (1.5 - 0.5 * m * y * y);
  y = y * (1.5 - 0.5 * m * y * y);
  return __builtin_bit_cast(double, __builtin_bit_cast(uint64_t, y) - ((uint64_t)h << 52));   // y * 2^-h
}
// QR of B (row c of B in thread c < 128, q; the other threads of the block hold zeros and keep them) by
// Gram-Schmidt applied twice; dependent columns become 0.  Called by all 256 threads.  The rows go
// through LDS (Bq) once; then each of the two waves that own rows holds ALL 128 rows, two per lane, and
// orthonormalises them by itself: every inner product is one reduction over the lanes of a wave, with no
// barrier and no LDS traffic (the two waves compute the same numbers in the same order and each keeps
// its own rows).
template <int R>
__device__ __forceinline__ void qr_columns(double (&q)[R], double (*Bq)[R] /* LDS [128][R] */) {
  const int c = threadIdx.x & (D - 1);
  const bool owner = threadIdx.x < D;
  block_lds_sync();
  if (owner) {
#pragma unroll
    for (int r = 0; r < R; ++r) Bq[c][r] = q[r];
  }
  block_lds_sync();
  if (!owner) return;   // (whole waves)
  const int lane = c & 63;
  double a[R], b[R];    // rows lane and lane + 64
#pragma unroll
  for (int r = 0; r < R; ++r) { a[r] = Bq[lane][r]; b[r] = Bq[lane + 64][r]; }
#pragma unroll
  for (int j = 0; j < R; ++j) {
    const double before2 = wave_sum_d(a[j] * a[j] + b[j] * b[j]);
    if (before2 == 0.0) { a[j] = 0.0; b[j] = 0.0; continue; }   // wave-uniform
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      double d[R];   // the projections of a pass are taken together (classical Gram-Schmidt, applied twice)
#pragma unroll
      for (int i = 0; i < R; ++i) d[i] = i < j ? wave_sum_d(a[i] * a[j] + b[i] * b[j]) : 0.0;
#pragma unroll
      for (int i = 0; i < R; ++i)
        if (i < j) { a[j] -= d[i] * a[i]; b[j] -= d[i] * b[i]; }
    }
    const double after2 = wave_sum_d(a[j] * a[j] + b[j] * b[j]);
    if (!(after2 > 1e-24 * before2)) { a[j] = 0.0; b[j] = 0.0; }   // norm after <= 1e-12 * norm before
    else {
      const double inv = rsqrt_d(after2);
      a[j] *= inv;
      b[j] *= inv;
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) q[r] = c < 64 ? a[r] : b[r];
}
// grid (B*H), block 256: thread (half = tid / 128, c = tid % 128).  Row c of B belongs to thread
// (0, c); the upper half of the block helps with the loads of G and with half of every product.
template <int R>
__global__ __launch_bounds__(256) void pi_solve_kernel(StartB sb, int rank,
                                                       const float* __restrict__ gram_partial, int nstrips, int rounds,
                                                       float* __restrict__ Bcur, int last_round, SegView sv) {
  GEAR_DYN_LDS(smem_raw);
  SolveSmem<R>& sm = *reinterpret_cast<SolveSmem<R>*>(smem_raw);
  const int slab = blockIdx.x, c = threadIdx.x & (D - 1), half = threadIdx.x >> 7;
  const bool owner = half == 0;
  if (rounds > 0) {
    // G = sum of the strips' partial tiles (fixed order): element tid + 256 j is register j % 4... of tile j
    const float* gp = gram_partial + (size_t)slab * nstrips * GRAM_FLOATS + threadIdx.x;
    float s[GRAM_TILES];
#pragma unroll
    for (int j = 0; j < GRAM_TILES; ++j) s[j] = 0.0f;
    for (int st = 0; st < nstrips; ++st) {
      float t[GRAM_TILES];   // a loop of their own for the loads: added into the sums directly, each would be waited for in turn
#pragma unroll
      for (int j = 0; j < GRAM_TILES; ++j) t[j] = __builtin_nontemporal_load(gp + (size_t)st * GRAM_FLOATS + 256 * j);
#pragma unroll
      for (int j = 0; j < GRAM_TILES; ++j) s[j] += t[j];
    }
    // element tid of tile (e, f): register i = tid / 64 of lane l = tid % 64, i.e. G[8*(4*(l/16)+i) + e][8*(l%16) + f]
    const int i = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int row0 = 8 * (4 * (l >> 4) + i), col0 = 8 * (l & 15);
    int j = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
      for (int f = e; f < 8; ++f) {
        sm.G[(row0 + e) * GP + col0 + f] = s[j];
        if (e != f) sm.G[(col0 + f) * GP + row0 + e] = s[j];   // a diagonal tile holds both (row, col) and (col, row) itself
        ++j;
      }
  }
  double q[R];
#pragma unroll
  for (int r = 0; r < R; ++r) q[r] = (owner && r < rank) ? (double)start_b(sb, slab, c, rank, r) : 0.0;
  for (int l = 0; l < rounds; ++l) {
    block_lds_sync();
    if (owner) {
#pragma unroll
      for (int r = 0; r < R; ++r) sm.Bs[c][r] = q[r];
    }
    block_lds_sync();
    double qn[R];
#pragma unroll
    for (int r = 0; r < R; ++r) qn[r] = 0.0;
#pragma unroll 8
    for (int k = 64 * half; k < 64 * half + 64; ++k) {
      const double gk = (double)sm.G[k * GP + c];   // G is symmetric: column c read as row-major neighbours
#pragma unroll
      for (int r = 0; r < R; ++r) qn[r] += gk * sm.Bs[k][r];
    }
    if (!owner) {
#pragma unroll
      for (int r = 0; r < R; ++r) sm.part[c][r] = (float)qn[r];
    }
    block_lds_sync();
#pragma unroll
    for (int r = 0; r < R; ++r) q[r] = owner ? qn[r] + sm.part[c][r] : 0.0;
    // keep magnitudes in range between rounds (unit columns: the next product stays far inside single
    // precision, which the upper half block's share passes through); after the last product the QR
    // below rescales anyway
    if (l + 1 < rounds) {   // block-uniform
      double n2[R];
#pragma unroll
      for (int r = 0; r < R; ++r) n2[r] = q[r] * q[r];
      block_sum_vec<R>(n2, sm.red);
#pragma unroll
      for (int r = 0; r < R; ++r) q[r] = n2[r] > 0.0 ? q[r] * rsqrt_d(n2[r]) : 0.0;
    }
  }
  qr_columns<R>(q, sm.Bs);
  if (!last_round) {
    if (owner) {
#pragma unroll
      for (int r = 0; r < R; ++r) Bcur[((size_t)slab * D + c) * R + r] = (float)q[r];
    }
    return;
  }
  // The last round of Algorithm 2 without another pass over R for B: with A = R B (B orthonormal now),
  // orth(A) = A C and the round's result B' = R^T orth(A) = (R^T R) B C = G B C, while the r x r Gram matrix
  // that gives C is A^T A = B^T G B.  What is left for the pass over R is A itself: orth(A) = R (B C), so
  // the projection matrix W = B C goes to Bcur and B' to the arena.
  block_lds_sync();
  if (owner) {
#pragma unroll
    for (int r = 0; r < R; ++r) sm.Bs[c][r] = q[r];
  }
  block_lds_sync();
  double pr[R];   // row c of P = G B
#pragma unroll
  for (int r = 0; r < R; ++r) pr[r] = 0.0;
#pragma unroll 8
  for (int k = 64 * half; k < 64 * half + 64; ++k) {
    const double gk = (double)sm.G[k * GP + c];
#pragma unroll
    for (int r = 0; r < R; ++r) pr[r] += gk * sm.Bs[k][r];
  }
  if (!owner) {
#pragma unroll
    for (int r = 0; r < R; ++r) sm.part[c][r] = (float)pr[r];
  }
  block_lds_sync();
#pragma unroll
  for (int r = 0; r < R; ++r) pr[r] = owner ? pr[r] + sm.part[c][r] : 0.0;
  block_lds_sync();
  if (owner) {   // the whole rows of P, next to those of B in LDS
#pragma unroll
    for (int r = 0; r < R; ++r) sm.part[c][r] = (float)pr[r];
  }
  block_lds_sync();
  if (threadIdx.x < R * R) {   // entry (i, j) of B^T P: one thread each (four running sums)
    const int i = threadIdx.x / R, j = threadIdx.x % R;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    for (int k = 0; k < D; k += 4) {
      s0 += sm.Bs[k][i] * sm.part[k][j];
      s1 += sm.Bs[k + 1][i] * sm.part[k + 1][j];
      s2 += sm.Bs[k + 2][i] * sm.part[k + 2][j];
      s3 += sm.Bs[k + 3][i] * sm.part[k + 3][j];
    }
    sm.C[i][j] = (s0 + s1) + (s2 + s3);
  }
  block_lds_sync();
  if (threadIdx.x < R * R) {   // symmetric up to rounding
    const int i = threadIdx.x / R, j = threadIdx.x % R;
    sm.GA[i][j] = 0.5 * (sm.C[i][j] + sm.C[j][i]);
  }
  block_lds_sync();
  if (threadIdx.x < 64) coeff_orth<R>(sm.GA, sm.C, sm.cj, (int)threadIdx.x);
  block_lds_sync();
  if (owner) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      double w = 0.0, bo = 0.0;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        w += q[r] * sm.C[r][j];
        bo += pr[r] * sm.C[r][j];
      }
      Bcur[((size_t)slab * D + c) * R + j] = (float)w;
      if (j < rank) sv.Bf[((size_t)slab * D + c) * sv.rank + j] = (uint16_t)f2h((float)bo);
    }
  }
}

// ------------------------------------------------------------------ segments of at most 64 tokens
// A flushed streaming buffer (n_b = 20 .. 64 tokens in the paper's settings) is small enough for one
// block to keep its residual in LDS: the rows are read and the residual derived once, and every round
// of Algorithm 2 runs out of LDS with a handful of block barriers; nothing goes through the workspace.
// Same steps and the same precision choices as the kernels above: A = R B and B' = R^T A accumulate in
// fp32, column scaling, the QR of B and the coefficient-space orth(A) in fp64.
// grid (B*H), block 256.  Thread (r0 = tid/16, oc = tid%16) derives channels 8*oc..+7 of rows
// r0 + 16 k and later forms their share of A; thread (half = tid/128, c = tid%128) sums rows
// [32 half, 32 half + 32) of B'[c][:], thread (0, c) owns row c of B.
constexpr int TINY_ROWS = 64;
constexpr int TINY_PITCH = D + 4;   // floats per residual row in LDS (16-byte aligned pieces)
template <int R>
struct TinySmem {
  __attribute__((aligned(16))) float Rs[TINY_ROWS][TINY_PITCH];   // rows >= n are 0
  __attribute__((aligned(16))) float Bs[D][R];
  float As[TINY_ROWS][R];
  float part[D][R];
  double Bq[D][R];      // the rows of B for its QR
  double red[4 * (R + 1)];
  double GA[R][R];
  double C[R][R];
  double cj[R];
};
template <bool IS_K, int R>
__global__ __launch_bounds__(256) void pi_tiny_kernel(const uint16_t* __restrict__ Y, SegView sv, int g, int bits, int n,
                                                      int t_lr, int iters, StartB sb) {
  __shared__ TinySmem<R> sm;
  const int slab = blockIdx.x, tid = threadIdx.x;
  const int r0 = tid >> 4, oc = tid & 15;
  const int c = tid & (D - 1), half = tid >> 7;
  const bool owner = half == 0;
  const int rank = sv.rank;
  // ---- the residual, once: R = (Y - zero) - code * scale (Keys: stored codes; Values: the quantizer's sequence)
  {
    const int lg = 31 - __clz(g), ngl = 7 - lg;   // (Keys with per-vector groups pass g = 32768: one group)
    const float qmax = (float)((1 << bits) - 1);
    const GEAR_BUF_T xbuf = GEAR_BUF_MAKE(Y + (size_t)slab * n * D, n * (D * 2));
    const GEAR_BUF_T cbuf = GEAR_BUF_MAKE(sv.codes + (size_t)slab * sv.n_cap * (4 * bits), IS_K ? n * (16 * bits) : 0);
    const GEAR_BUF_T pbuf = IS_K ? GEAR_BUF_MAKE(sv.sz + (size_t)slab * sv.ng_cap * D, ((n + g - 1) >> lg) * (D * 4))
                                 : GEAR_BUF_MAKE(sv.sz + (((size_t)slab * sv.n_cap) << ngl), (n << ngl) * 4);
    uint4 xv[4], pz[2][2];
    uint32_t cw[4], pv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {   // every load is requested before the first one is used
      const int t = r0 + 16 * k;
      xv[k] = GEAR_BUF_LOAD16_NT(xbuf, t * (D * 2) + oc * 16);   // rows past the end read as 0
      cw[k] = 0u;
      pv[k] = 0u;
      if (IS_K) {
        const int co = t * (16 * bits) + oc * (bits == 4 ? 4 : 2);
        cw[k] = bits == 4 ? GEAR_BUF_LOAD4(cbuf, co) : GEAR_BUF_LOAD2(cbuf, co);
      } else {
        pv[k] = GEAR_BUF_LOAD4(pbuf, ((t << ngl) + ((oc * 8) >> lg)) * 4);
      }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {   // Keys: 64 rows lie in at most two groups (g >= 32)
      pz[j][0] = make_uint4(0, 0, 0, 0);
      pz[j][1] = make_uint4(0, 0, 0, 0);
      if (IS_K) {
        pz[j][0] = GEAR_BUF_LOAD16(pbuf, (j * D + oc * 8) * 4);
        pz[j][1] = GEAR_BUF_LOAD16(pbuf, (j * D + oc * 8) * 4 + 16);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int t = r0 + 16 * k;
      const uint32_t w[4] = {xv[k].x, xv[k].y, xv[k].z, xv[k].w};
      float res[8];
      if (IS_K) {
        const bool second = (t >> lg) != 0;
        const uint4 z0 = second ? pz[1][0] : pz[0][0], z1 = second ? pz[1][1] : pz[0][1];
        const uint32_t z[8] = {z0.x, z0.y, z0.z, z0.w, z1.x, z1.y, z1.z, z1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = h2f((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
          res[e] = __builtin_fmaf(-(float)GEAR_UBFE(cw[k], e * bits, bits), h2f(z[e] & 0xFFFFu), y - h2f(z[e] >> 16));
        }
      } else {
        const GroupQ q = load_group(pv[k]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float y = h2f((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xFFFFu));
          res[e] = quant_error(y, q.mn, q.inv, q.delta, qmax);
        }
      }
      if (t >= n || t < t_lr) {   // no such row / a row that takes no part in the low-rank term
#pragma unroll
        for (int e = 0; e < 8; ++e) res[e] = 0.0f;
      }
      *reinterpret_cast<float4*>(&sm.Rs[t][oc * 8]) = make_float4(res[0], res[1], res[2], res[3]);
      *reinterpret_cast<float4*>(&sm.Rs[t][oc * 8 + 4]) = make_float4(res[4], res[5], res[6], res[7]);
    }
  }
  double q[R];
#pragma unroll
  for (int r = 0; r < R; ++r) q[r] = (owner && r < rank) ? (double)start_b(sb, slab, c, rank, r) : 0.0;
  if (iters == 1) qr_columns<R>(q, sm.Bq);   // the only round is also the last: B is orthonormalised first
#pragma unroll 1
  for (int l = 0; l < iters; ++l) {
    const bool last = l == iters - 1;
    block_lds_sync();
    if (owner) {
#pragma unroll
      for (int r = 0; r < R; ++r) sm.Bs[c][r] = (float)q[r];
    }
    block_lds_sync();
    // A = R B: the 16 lanes of a row of lanes hold one token
    {
      float bc[8][R];
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int r = 0; r < R; ++r) bc[e][r] = sm.Bs[oc * 8 + e][r];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (16 * k >= n) break;   // block-uniform
        const int t = r0 + 16 * k;
        const float4 x0 = *reinterpret_cast<const float4*>(&sm.Rs[t][oc * 8]);
        const float4 x1 = *reinterpret_cast<const float4*>(&sm.Rs[t][oc * 8 + 4]);
        const float res[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
        for (int r = 0; r < R; ++r) {
          float a = 0.0f;
#pragma unroll
          for (int e = 0; e < 8; ++e) a += res[e] * bc[e][r];
          a = row16_sum(a);
          if (oc == 0) sm.As[t][r] = a;
        }
      }
    }
    block_lds_sync();
    // B' = R^T A
    float p[R];
#pragma unroll
    for (int r = 0; r < R; ++r) p[r] = 0.0f;
    {
      const int t_hi = n < 32 * half + 32 ? n : 32 * half + 32;
      for (int t = 32 * half; t < t_hi; ++t) {
        const float rv = sm.Rs[t][c];
#pragma unroll
        for (int r = 0; r < R; ++r) p[r] += rv * sm.As[t][r];
      }
    }
    if (!owner) {
#pragma unroll
      for (int r = 0; r < R; ++r) sm.part[c][r] = p[r];
    }
    block_lds_sync();
    double qn[R];
#pragma unroll
    for (int r = 0; r < R; ++r) qn[r] = owner ? (double)p[r] + (double)sm.part[c][r] : 0.0;
    if (!last) {
      // keep magnitudes in range between rounds (the span, hence A B^T, is unchanged)
      double n2[R];
#pragma unroll
      for (int r = 0; r < R; ++r) n2[r] = qn[r] * qn[r];
      block_sum_vec<R>(n2, sm.red);
#pragma unroll
      for (int r = 0; r < R; ++r) q[r] = n2[r] > 0.0 ? qn[r] * rsqrt_d(n2[r]) : 0.0;
      if (l == iters - 2) qr_columns<R>(q, sm.Bq);   // the QR of B that opens the last round
      continue;
    }
    // last round: orth(A) = A C from the r x r Gram matrix of A; B = R^T orth(A) = B' C
    if (tid < R * R) {
      const int i = tid / R, j = tid % R;
      double s = 0.0;
      for (int t = 0; t < n; ++t) s += (double)sm.As[t][i] * (double)sm.As[t][j];
      sm.GA[i][j] = s;
    }
    block_lds_sync();
    if (tid < 64) coeff_orth<R>(sm.GA, sm.C, sm.cj, tid);
    block_lds_sync();
    if (owner) {
      for (int j = 0; j < rank; ++j) {
        double bo = 0.0;
#pragma unroll
        for (int r = 0; r < R; ++r) bo += qn[r] * sm.C[r][j];
        sv.Bf[((size_t)slab * D + c) * rank + j] = (uint16_t)f2h((float)bo);
      }
    }
    for (int i = tid; i < n * rank; i += 256) {
      const int t = i / rank, j = i - t * rank;
      float a = 0.0f;
#pragma unroll
      for (int r = 0; r < R; ++r) a += sm.As[t][r] * (float)sm.C[r][j];
      sv.A[((size_t)slab * sv.n_cap + t) * rank + j] = (uint16_t)f2h(a);
    }
  }
}

// ------------------------------------------------------------------ host side
// Tokens per strip of the Gram pass: the longest that still gives every resident block slot (two per CU,
// 512 on the chip) a strip; the solve kernel, one block per slab, then has the fewest partials to add.
int pi_gram_strip(int n, int slabs) {
  for (int strip = 2048; strip > 512; strip >>= 1)
    if ((long long)slabs * ((n + strip - 1) / strip) >= 512) return strip;
  return 512;
}
int pi_gram_strips_max(int n_max, int slabs) {
  const int m = (1024 + slabs - 1) / slabs;   // strips per slab that fill the chip
  const int coarse = (n_max + 2047) / 2048, fine = (n_max + 511) / 512;
  const int want = 2 * m > coarse ? 2 * m : coarse;
  return want < fine ? want : fine;
}

template <bool IS_K, int LG>
static void launch_gram(const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int t_lr, int strip, int nstrips, float* gram,
                        hipStream_t st) {
  // (per-vector grouping: the one Key group of a segment is addressed as a group of 32768 tokens)
  hipLaunchKernelGGL((pi_gram_kernel<IS_K, LG>), dim3(nstrips, dm.B * dm.H), dim3(256), 0, st, Yf, sv, IS_K ? 1 << LG : dm.g, dm.bits, n, t_lr, strip, gram);
}

template <int R>
static hipError_t run_pi(bool is_k, const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int t_lr, int iters,
                         StartB sb, float* Bcur, float* partial, float* Atmp, float* cmat, float* gram,
                         int gram_strips_cap, hipStream_t st) {
  const int slabs = dm.B * dm.H;
  const int npart = (n + PT - 1) / PT;
  const int g_eff = (is_k && dm.kcvt) ? 32768 : dm.g;   // per-vector grouping: one Key group per segment
  if (npart == 1) {   // a short segment: everything in one block per slab
    if (n <= TINY_ROWS) {   // (a flushed buffer of the paper's sizes) with its residual resident in LDS
      if (is_k)
        hipLaunchKernelGGL((pi_tiny_kernel<true, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, g_eff, dm.bits, n, t_lr, iters, sb);
      else
        hipLaunchKernelGGL((pi_tiny_kernel<false, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, t_lr, iters, sb);
      return hipGetLastError();
    }
    if (is_k)
      hipLaunchKernelGGL((pi_small_kernel<true, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, g_eff, dm.bits, n, t_lr, iters, sb, Bcur, partial, Atmp, cmat);
    else
      hipLaunchKernelGGL((pi_small_kernel<false, R>), dim3(slabs), dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, t_lr, iters, sb, Bcur, partial, Atmp, cmat);
    return hipGetLastError();
  }
  // rounds 1 .. L-1: B <- (R^T R)^(L-1) B0 from one pass that forms the Gram matrix; then QR(B)
  int nstrips = 0;
  if (iters > 1) {
    const int strip = pi_gram_strip(n, slabs);
    nstrips = (n + strip - 1) / strip;
    if (nstrips > gram_strips_cap) return hipErrorInvalidValue;
    if (!is_k) launch_gram<false, 0>(Yf, sv, dm, n, t_lr, strip, nstrips, gram, st);
    else if (dm.kcvt) launch_gram<true, 15>(Yf, sv, dm, n, t_lr, strip, nstrips, gram, st);
    else if (dm.g == 32) launch_gram<true, 5>(Yf, sv, dm, n, t_lr, strip, nstrips, gram, st);
    else if (dm.g == 64) launch_gram<true, 6>(Yf, sv, dm, n, t_lr, strip, nstrips, gram, st);
    else launch_gram<true, 7>(Yf, sv, dm, n, t_lr, strip, nstrips, gram, st);
  }
  {
    static std::atomic<bool> lds_raised{false};   // per kernel instance (R); two threads may both raise it: harmless
    if (!lds_raised.load(std::memory_order_relaxed)) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(pi_solve_kernel<R>),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(SolveSmem<R>));
      if (e != hipSuccess) return e;
      lds_raised.store(true, std::memory_order_relaxed);
    }
  }
  hipLaunchKernelGGL(pi_solve_kernel<R>, dim3(slabs), dim3(256), sizeof(SolveSmem<R>), st, sb, sv.rank, (const float*)gram,
                     nstrips, iters - 1, Bcur, iters > 1 ? 1 : 0, sv);
  if (iters > 1) {
    // the last round's B and the factor of orth(A) came out of the Gram matrix; one light pass writes A
    const dim3 grid(npart, slabs);
    if (is_k)
      hipLaunchKernelGGL((pi_project_kernel<true, R>), grid, dim3(256), 0, st, Yf, sv, g_eff, dm.bits, n, t_lr, (const float*)Bcur);
    else
      hipLaunchKernelGGL((pi_project_kernel<false, R>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, t_lr, (const float*)Bcur);
    return hipGetLastError();
  }
  // a single round (no Gram pass): A = R B, orth(A) through its r x r Gram matrix, B = R^T A
  {
    const dim3 grid(npart, slabs);
    if (is_k)
      hipLaunchKernelGGL((pi_sweep_kernel<true, R, true>), grid, dim3(256), 0, st, Yf, sv, g_eff, dm.bits, n, t_lr, (const float*)Bcur, partial, npart, Atmp);
    else
      hipLaunchKernelGGL((pi_sweep_kernel<false, R, true>), grid, dim3(256), 0, st, Yf, sv, dm.g, dm.bits, n, t_lr, (const float*)Bcur, partial, npart, Atmp);
    hipLaunchKernelGGL(pi_update_kernel<R>, dim3(slabs), dim3(256), 0, st, 0, sb, sv.rank,
                       (const float*)partial, npart, 0, 1, Bcur, cmat, sv);
  }
  hipLaunchKernelGGL(pi_finish_kernel<R>, dim3((n + 255) / 256, slabs), dim3(256), 0, st, (const float*)Atmp,
                     (const float*)cmat, sv, n);
  return hipGetLastError();
}

int pi_padded_rank(int rank) { return rank <= 2 ? 2 : rank <= 4 ? 4 : 8; }

hipError_t launch_power_iteration(bool is_k, const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int t_lr, int iters,
                                  const float* init_B, uint64_t seed, float* Bcur, float* partial, float* Atmp, float* cmat,
                                  float* gram, int gram_strips_cap, hipStream_t st) {
  // this tensor's part of the [2 (K, V), B, H, 128, rank] start array
  const uint64_t tensor_entries = (uint64_t)dm.B * dm.H * D * sv.rank;
  const StartB sb{init_B ? init_B + (is_k ? 0 : tensor_entries) : nullptr, seed, is_k ? 0 : tensor_entries};
  switch (pi_padded_rank(sv.rank)) {
    case 2: return run_pi<2>(is_k, Yf, sv, dm, n, t_lr, iters, sb, Bcur, partial, Atmp, cmat, gram, gram_strips_cap, st);
    case 4: return run_pi<4>(is_k, Yf, sv, dm, n, t_lr, iters, sb, Bcur, partial, Atmp, cmat, gram, gram_strips_cap, st);
    default: return run_pi<8>(is_k, Yf, sv, dm, n, t_lr, iters, sb, Bcur, partial, Atmp, cmat, gram, gram_strips_cap, st);
  }
}

}  // namespace gear
