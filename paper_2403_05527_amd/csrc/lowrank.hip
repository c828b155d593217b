// SVDSolver_r (Eq. 6, Algorithm 2): batched power iteration on the per-head
// residual R = X - D - S, which the quantization kernels leave in a workspace
// buffer as the rounding remainder u = R / scale in 24-bit fixed point (|u| <= 1/2,
// i.e. fp32's own precision in 3 bytes per entry; a 16-bit copy flips too many
// fp16 roundings of the stored factors against a double-precision computation).
//
//   pi_update  : B <- start matrix or sum of the sweep partials; column scaling
//                between rounds (the span, hence A B^T, is unchanged); QR of B
//                before the last round; after the last round the r x r factor
//                that orthonormalises A, and the final B = R^T orth(A).
//   pi_sweep   : one pass over a slab's residual: a_t = R_t B (per token), partial
//                B' = sum_t R_t^T a_t, and in the last round a_t itself and the
//                Gram matrix sum_t a_t a_t^T.
//   pi_finish  : A = a C  (C = the r x r factor), rounded to fp16.
#include "gear_internal.h"
#include "gear_launch.h"

namespace gear {

constexpr int PT = 256;  // tokens per sweep block
constexpr float RESID_UNIT = 1.0f / 2147483648.0f;   // 2^-31: the stored remainder is read as an integer times 2^8

template <typename T>
__device__ __forceinline__ T block128_sum(T v, T* red /* >= 2 */) {
  v = wave_sum_shfl(v);
  block_lds_sync();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  block_lds_sync();
  return red[0] + red[1];
}

// grid (B*H), block 128: thread c owns row c of the [128 x R] matrix.
// src_init != nullptr : B <- init (fp32 [slab][128][rank], zero-padded to R)
// else                : B <- sum over `npart` partials ([slab][npart][128*R + R*R])
// do_orth : replace B by the Q factor of its QR (twice-applied modified
//           Gram-Schmidt, fp64; dependent columns become 0)
// final   : also sum the Gram partials, build C with orth(A) = A C, write
//           B_out = B C as fp16 into the arena and C into cmat.
template <int R>
__global__ __launch_bounds__(128) void pi_update_kernel(const float* __restrict__ src_init, int rank,
                                                        const float* __restrict__ partial, int npart,
                                                        int do_orth, int final_round,
                                                        float* __restrict__ Bcur, float* __restrict__ cmat,
                                                        SegView sv) {
  __shared__ double red[2];
  __shared__ double G[R][R];
  __shared__ double C[R][R];
  const int slab = blockIdx.x, c = threadIdx.x;
  double q[R];
  if (src_init) {
#pragma unroll
    for (int r = 0; r < R; ++r) q[r] = r < rank ? (double)src_init[((size_t)slab * D + c) * rank + r] : 0.0;
  } else {
#pragma unroll
    for (int r = 0; r < R; ++r) q[r] = 0.0;
    const float* p = partial + (size_t)slab * npart * (D * R + R * R);
    for (int i = 0; i < npart; ++i) {
#pragma unroll
      for (int r = 0; r < R; ++r) q[r] += (double)p[(size_t)i * (D * R + R * R) + c * R + r];
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
      bool valid[R];
      for (int j = 0; j < R; ++j) {
        double cj[R];
        for (int i = 0; i < R; ++i) cj[i] = (i == j) ? 1.0 : 0.0;
        const double before2 = G[j][j];
        valid[j] = before2 > 0.0;
        if (valid[j]) {
          for (int pass = 0; pass < 2; ++pass)
            for (int k = 0; k < j; ++k) {
              if (!valid[k]) continue;
              double dot = 0.0;  // q_k^T v = c_k^T G c_j
              for (int a = 0; a < R; ++a)
                for (int b = 0; b < R; ++b) dot += C[a][k] * G[a][b] * cj[b];
              for (int a = 0; a < R; ++a) cj[a] -= dot * C[a][k];
            }
          double after2 = 0.0;
          for (int a = 0; a < R; ++a)
            for (int b = 0; b < R; ++b) after2 += cj[a] * G[a][b] * cj[b];
          if (!(after2 > 1e-10 * before2)) valid[j] = false;
          else {
            const double inv = 1.0 / sqrt(after2);
            for (int a = 0; a < R; ++a) cj[a] *= inv;
          }
        }
        for (int a = 0; a < R; ++a) C[a][j] = valid[j] ? cj[a] : 0.0;
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
    for (int j = 0; j < rank; ++j) sv.Bf[((size_t)slab * D + c) * sv.rank + j] = (uint16_t)f2h((float)o[j]);
    if (c < R * R) cmat[(size_t)slab * R * R + c] = (float)C[c / R][c % R];
    return;
  }

  if (do_orth) {
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const double before2 = block128_sum(q[j] * q[j], red);
      if (before2 == 0.0) { q[j] = 0.0; continue; }
      for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
          if (i < j) {
            const double dot = block128_sum(q[i] * q[j], red);
            q[j] -= dot * q[i];
          }
        }
      }
      const double after2 = block128_sum(q[j] * q[j], red);
      if (!(sqrt(after2) > 1e-12 * sqrt(before2))) q[j] = 0.0;
      else q[j] *= 1.0 / sqrt(after2);
    }
  } else {
    // keep magnitudes in range between rounds
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const double n2 = block128_sum(q[j] * q[j], red);
      if (n2 > 0.0) q[j] *= 1.0 / sqrt(n2);
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) Bcur[((size_t)slab * D + c) * R + r] = (float)q[r];
}

// grid (ceil(n/PT), B*H), block 256; thread (r0 = tid/16, oc = tid%16) owns
// channels 8*oc..+7 of rows pt*PT + r0 + 16*k of the stored residual
// (u = R / scale as 16-bit fixed point; the scale is applied per group here).
// LAST: the final round, which also leaves a_t and the Gram matrix (its extra state costs
// one resident block per CU, so the rounds before it are compiled without).
template <bool IS_K, int R, bool LAST>
__global__ __launch_bounds__(256, (R <= 2 ? 4 : R <= 4 ? 3 : 2)) void pi_sweep_kernel(const uint16_t* __restrict__ Rres,
                                                       const uint8_t* __restrict__ Rlo, SegView sv, int g, int n,
                                                       const float* __restrict__ Bcur,
                                                       float* __restrict__ partial, int npart,
                                                       float* __restrict__ Atmp) {
  __shared__ float red[4][D * R];
  __shared__ float redg[4][R * R];
  const int slab = blockIdx.y, pt = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r0 = tid >> 4, oc = tid & 15;
  const uint16_t* Xs = Rres + (size_t)slab * n * D;
  const uint8_t* Xl = Rlo + (size_t)slab * n * D;
  const int lg = 31 - __clz(g);   // g is a power of two

  float bc[8][R];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int r = 0; r < R; ++r) bc[e][r] = Bcur[((size_t)slab * D + oc * 8 + e) * R + r];

  float acc[8][R];
  float gacc[R];
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int r = 0; r < R; ++r) acc[e][r] = 0.0f;
#pragma unroll
  for (int r = 0; r < R; ++r) gacc[r] = 0.0f;

  constexpr int UN = 4;  // rows in flight per thread
  for (int k0 = 0; k0 < PT / 16; k0 += UN) {
    if (pt * PT + 16 * k0 >= n) break;  // block-uniform
    uint4 xv[UN];
    uint2 xl[UN];
    // Keys: the UN = 4 bands of 16 rows in flight lie in one group (g >= 64) or two (g = 32),
    // so at most two sets of per-channel scales are needed
    const int ush = g >= 64 ? 2 : 1;                 // band u uses scale set u >> ush
    uint4 sk0[IS_K ? 2 : 1], sk1[IS_K ? 2 : 1];     // raw (scale, zero) words, Keys
    uint32_t svw[UN];                               // raw (scale, zero) word, Values
    // every load of the UN rows is issued before the first result is touched
    if (IS_K) {
#pragma unroll
      for (int gs = 0; gs < 2; ++gs) {
        const int t = pt * PT + 16 * (k0 + (gs << ush));       // first row of the set's first band
        sk0[gs] = make_uint4(0, 0, 0, 0);
        sk1[gs] = make_uint4(0, 0, 0, 0);
        if ((gs << ush) < UN && t < n) {
          const uint4* p = reinterpret_cast<const uint4*>(sv.sz + ((size_t)slab * sv.ng_cap + (t >> lg)) * D + oc * 8);
          sk0[gs] = p[0];
          sk1[gs] = p[1];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int t = pt * PT + r0 + 16 * (k0 + u);
      xv[u] = make_uint4(0, 0, 0, 0);
      xl[u] = make_uint2(0, 0);
      svw[u] = 0u;
      if (t < n) {
        xv[u] = load_stream16(Xs + (size_t)t * D + oc * 8);
        xl[u] = load_stream8(Xl + (size_t)t * D + oc * 8);
        if (!IS_K)   // scale of (token t, the channel group of my 8 channels)
          svw[u] = sv.sz[((size_t)slab * sv.n_cap + t) * (D >> lg) + ((oc * 8) >> lg)];
      }
    }
    float dlk[IS_K ? 2 : 1][IS_K ? 8 : 1], dlv[UN];
    if (IS_K) {
#pragma unroll
      for (int gs = 0; gs < 2; ++gs) {
        const uint32_t sb[8] = {sk0[gs].x, sk0[gs].y, sk0[gs].z, sk0[gs].w, sk1[gs].x, sk1[gs].y, sk1[gs].z, sk1[gs].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) dlk[gs][IS_K ? e : 0] = h2f(sb[e] & 0xFFFFu) * RESID_UNIT;
      }
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) dlv[u] = h2f(svw[u] & 0xFFFFu) * RESID_UNIT;
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int t = pt * PT + r0 + 16 * (k0 + u);
      const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
      const uint32_t wl[2] = {xl[u].x, xl[u].y};
      // the remainder times 2^31 (exact), times the scale with the 2^-31 folded in
      float res[8];
      float a[R];
#pragma unroll
      for (int r = 0; r < R; ++r) a[r] = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        res[e] = resid_x2p31(w[e >> 1], wl[e >> 2], e) * (IS_K ? dlk[IS_K ? ((u >> ush) & 1) : 0][IS_K ? e : 0] : dlv[u]);
#pragma unroll
        for (int r = 0; r < R; ++r) a[r] += res[e] * bc[e][r];
      }
#pragma unroll
      for (int r = 0; r < R; ++r) a[r] = row16_sum(a[r]);   // the 16 lanes of a row hold one token
#pragma unroll
      for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[e][r] += res[e] * a[r];
      if (LAST) {
        if (oc == 0 && t < n) {
#pragma unroll
          for (int r = 0; r < R; ++r) Atmp[((size_t)slab * n + t) * R + r] = a[r];
        }
        if (oc < R) {
          float mine = 0.0f;
#pragma unroll
          for (int r = 0; r < R; ++r) mine = (r == oc) ? a[r] : mine;
#pragma unroll
          for (int r = 0; r < R; ++r) gacc[r] += mine * a[r];
        }
      }
    }
  }

  // reduce over the 16 row-threads that share a channel octet
#pragma unroll
  for (int e = 0; e < 8; ++e)
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float v = acc[e][r];
      v += __shfl_xor(v, 16, 64);
      v += __shfl_xor(v, 32, 64);
      acc[e][r] = v;
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
      for (int r = 0; r < R; ++r) red[wave][(oc * 8 + e) * R + r] = acc[e][r];
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

// grid (ceil(n/256), B*H), block 256: one token per thread.
template <int R>
__global__ __launch_bounds__(256) void pi_finish_kernel(const float* __restrict__ Atmp,
                                                        const float* __restrict__ cmat, SegView sv, int n) {
  __shared__ float C[R * R];
  const int slab = blockIdx.y;
  if (threadIdx.x < R * R) C[threadIdx.x] = cmat[(size_t)slab * R * R + threadIdx.x];
  block_lds_sync();
  const int t = blockIdx.x * 256 + threadIdx.x;
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

// ------------------------------------------------------------------ host side
template <int R>
static hipError_t run_pi(bool is_k, const uint16_t* Rres, const uint8_t* Rlo, const SegView& sv, const Dims& dm, int n, int iters,
                         const float* init_B, float* Bcur, float* partial, float* Atmp, float* cmat,
                         hipStream_t st) {
  const int slabs = dm.B * dm.H;
  const int npart = (n + PT - 1) / PT;
  hipLaunchKernelGGL(pi_update_kernel<R>, dim3(slabs), dim3(128), 0, st, init_B, sv.rank, (const float*)nullptr,
                     0, iters == 1 ? 1 : 0, 0, Bcur, cmat, sv);
  for (int l = 0; l < iters; ++l) {
    const int last = (l == iters - 1);
    const dim3 grid(npart, slabs);
    if (is_k && last)
      hipLaunchKernelGGL((pi_sweep_kernel<true, R, true>), grid, dim3(256), 0, st, Rres, Rlo, sv, dm.g, n, (const float*)Bcur, partial, npart, Atmp);
    else if (is_k)
      hipLaunchKernelGGL((pi_sweep_kernel<true, R, false>), grid, dim3(256), 0, st, Rres, Rlo, sv, dm.g, n, (const float*)Bcur, partial, npart, Atmp);
    else if (last)
      hipLaunchKernelGGL((pi_sweep_kernel<false, R, true>), grid, dim3(256), 0, st, Rres, Rlo, sv, dm.g, n, (const float*)Bcur, partial, npart, Atmp);
    else
      hipLaunchKernelGGL((pi_sweep_kernel<false, R, false>), grid, dim3(256), 0, st, Rres, Rlo, sv, dm.g, n, (const float*)Bcur, partial, npart, Atmp);
    hipLaunchKernelGGL(pi_update_kernel<R>, dim3(slabs), dim3(128), 0, st, (const float*)nullptr, sv.rank,
                       (const float*)partial, npart, (l == iters - 2) ? 1 : 0, last, Bcur, cmat, sv);
  }
  hipLaunchKernelGGL(pi_finish_kernel<R>, dim3((n + 255) / 256, slabs), dim3(256), 0, st, (const float*)Atmp,
                     (const float*)cmat, sv, n);
  return hipGetLastError();
}

int pi_padded_rank(int rank) { return rank <= 2 ? 2 : rank <= 4 ? 4 : 8; }

hipError_t launch_power_iteration(bool is_k, const uint16_t* Rres, const uint8_t* Rlo, const SegView& sv, const Dims& dm, int n, int iters,
                                  const float* init_B, float* Bcur, float* partial, float* Atmp, float* cmat,
                                  hipStream_t st) {
  switch (pi_padded_rank(sv.rank)) {
    case 2: return run_pi<2>(is_k, Rres, Rlo, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
    case 4: return run_pi<4>(is_k, Rres, Rlo, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
    default: return run_pi<8>(is_k, Rres, Rlo, sv, dm, n, iters, init_B, Bcur, partial, Atmp, cmat, st);
  }
}

}  // namespace gear
