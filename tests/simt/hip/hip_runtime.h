// CPU stand-in for <hip/hip_runtime.h>, for tests only: it lets the library's .hip
// sources be compiled as plain C++ by the host compiler and run under the address,
// thread and memory sanitizers.  A kernel launch runs its grid one block at a time
// with one OS thread per work-item; the cross-lane operations the kernels use
// (DPP, readlane, shuffles, ballot, the 16x16x32 fp16 MFMA) exchange data through
// per-wave slots and pthread barriers; a wave-level barrier is a real barrier, so a
// kernel that relies on lock-step execution where it has no barrier shows up as a
// data race.  Statically sized LDS lives in one ELF section and is refilled with
// garbage before every block, dynamically sized LDS is an exact-size heap block.
#pragma once
#include <pthread.h>
#include <stdint.h>
#include <string.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <algorithm>
using std::min;
using std::max;
#define __device__
#define __host__
#define __global__
#define __forceinline__ inline
#define __launch_bounds__(...)
// all statically sized LDS lands in one ELF section, which the runtime fills with garbage before every block
#define __shared__ static __attribute__((section("simt_lds")))
#define __align__(n) __attribute__((aligned(n)))
struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };
struct uint2 { uint32_t x, y; };
struct alignas(16) uint4 { uint32_t x, y, z, w; };
struct alignas(16) float4 { float x, y, z, w; };
struct float2 { float x, y; };
static inline float4 make_float4(float x, float y, float z, float w) { return float4{x, y, z, w}; }
static inline float2 make_float2(float x, float y) { return float2{x, y}; }
static inline uint2 make_uint2(uint32_t x, uint32_t y) { return uint2{x, y}; }
static inline uint4 make_uint4(uint32_t x, uint32_t y, uint32_t z, uint32_t w) { return uint4{x, y, z, w}; }
struct simt_buf;
template <typename T> static inline T simt_buf_load(const simt_buf& b, uint32_t off);
typedef int hipError_t;
typedef void* hipStream_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1 };
enum { hipFuncAttributeMaxDynamicSharedMemorySize = 8 };
inline hipError_t hipGetLastError() { return hipSuccess; }
inline hipError_t hipFuncSetAttribute(const void*, int, int) { return hipSuccess; }
inline const char* hipGetErrorString(hipError_t) { return "emulated"; }
inline hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
#define HIP_SYMBOL(x) x
inline hipError_t hipGetSymbolAddress(void** p, const void* sym) { *p = const_cast<void*>(sym); return hipSuccess; }
#define GEAR_DYN_LDS(name) unsigned char* name = simt::dyn_lds
#define GEAR_PIN_VGPR(x) asm volatile("" : "+r"(x))
#define GEAR_LDS_BARRIER() pthread_barrier_wait(&simt::block_bar)
#define GEAR_WAVE_UNIFORM(x) (x)
#define GEAR_BYTE_PERM(hi, lo, sel) simt_byte_perm((hi), (lo), (sel))
#define GEAR_FMED3(x, lo, hi) fminf(fmaxf((x), (lo)), (hi))
#define GEAR_UBFE(x, off, width) (((uint32_t)(x) >> (off)) & ((1u << (width)) - 1u))
struct simt_buf { const unsigned char* p; uint32_t n; };
#define GEAR_BUF_T simt_buf
#define GEAR_BUF_MAKE(p, bytes) simt_buf{reinterpret_cast<const unsigned char*>(p), (uint32_t)(bytes)}
#define GEAR_BUF_LOAD8(b, off) simt_buf_load<uint2>((b), (uint32_t)(off))
#define GEAR_BUF_LOAD16(b, off) simt_buf_load<uint4>((b), (uint32_t)(off))
#define GEAR_BUF_LOAD16_NT(b, off) simt_buf_load<uint4>((b), (uint32_t)(off))
#define GEAR_BUF_LOAD4(b, off) simt_buf_load<uint32_t>((b), (uint32_t)(off))
#define GEAR_BUF_LOAD2(b, off) ((uint32_t)simt_buf_load<uint16_t>((b), (uint32_t)(off)))
#define GEAR_BUF_STORE16_NT(b, off, v) simt_buf_store((b), (uint32_t)(off), (v))
#define GEAR_BUF_STORE4(b, off, v) simt_buf_store<uint32_t>((b), (uint32_t)(off), (uint32_t)(v))
#define GEAR_BUF_STORE2(b, off, v) simt_buf_store<uint16_t>((b), (uint32_t)(off), (uint16_t)(v))
// a store that does not lie wholly inside the view is dropped
template <typename T> static inline void simt_buf_store(const simt_buf& b, uint32_t off, const T& v) {
  if ((uint64_t)off + sizeof(T) <= b.n) memcpy(const_cast<unsigned char*>(b.p) + off, &v, sizeof(T));
}
// a load that does not lie wholly inside the view returns 0
template <typename T> static inline T simt_buf_load(const simt_buf& b, uint32_t off) {
  T r;
  memset(&r, 0, sizeof(T));
  if ((uint64_t)off + sizeof(T) <= b.n) memcpy(&r, b.p + off, sizeof(T));
  return r;
}
static inline uint32_t simt_byte_perm(uint32_t hi, uint32_t lo, uint32_t sel) {
  const uint64_t src = ((uint64_t)hi << 32) | lo;
  uint32_t r = 0;
  for (int i = 0; i < 4; ++i) {
    const uint32_t s = (sel >> (8 * i)) & 0xFFu;
    const uint32_t b = s < 8 ? (uint32_t)((src >> (8 * s)) & 0xFFu) : 0u;   // 0x0c: zero
    r |= b << (8 * i);
  }
  return r;
}
extern thread_local dim3 threadIdx;
extern thread_local dim3 blockIdx;
extern dim3 blockDim, gridDim;

namespace simt {
struct Wave {
  pthread_barrier_t bar;
  uint64_t slot[64];
  _Float16 ma[64][8], mb[64][8];
};
extern Wave waves[16];
extern pthread_barrier_t block_bar;
inline int lane() { return threadIdx.x & 63; }
inline Wave& W() { return waves[threadIdx.x >> 6]; }
inline void wave_barrier() { pthread_barrier_wait(&W().bar); }
inline uint64_t xchg(uint64_t v, int src) {
  Wave& w = W();
  w.slot[lane()] = v;
  pthread_barrier_wait(&w.bar);
  const uint64_t r = w.slot[src & 63];
  pthread_barrier_wait(&w.bar);
  return r;
}
inline int dpp_src(int l, int ctrl) {
  const int row = l & ~15, i = l & 15;
  if (ctrl < 0x100) {  // quad_perm
    const int q = l & ~3, j = l & 3;
    return q + ((ctrl >> (2 * j)) & 3);
  }
  if (ctrl == 0x140) return row + (15 - i);            // row_mirror
  if (ctrl == 0x141) return (l & ~7) + (7 - (l & 7));  // row_half_mirror
  if (ctrl > 0x120 && ctrl <= 0x12F) return row + ((i - (ctrl & 15)) & 15);  // row_ror:n
  fprintf(stderr, "dpp ctrl %x not modelled\n", ctrl);
  abort();
}
inline int dpp(int v, int ctrl) { return (int)(uint32_t)xchg((uint32_t)v, dpp_src(lane(), ctrl)); }
// with a row mask: rows outside it keep `old`; row_bcast:15 (0x142) gives rows 1..3 lane 15 of the row before,
// row_bcast:31 (0x143) gives rows 2, 3 lane 31; lanes without a source keep `old`
// row_shl:n (0x101..0x10F): lane i of a row reads lane i + n; row_shr:n (0x111..0x11F): lane i - n; a lane whose
// source lies outside the row reads 0 with bound_ctrl, else keeps `old`
inline int dpp_rows(int old, int v, int ctrl, int row_mask, bool bound_ctrl = false) {
  const int l = lane(), row = l >> 4, i = l & 15;
  int src = l;
  bool enabled = ((row_mask >> row) & 1) != 0, valid = true;
  if (ctrl == 0x142) { valid = row >= 1; src = row * 16 - 1; }
  else if (ctrl == 0x143) { valid = row >= 2; src = 31; }
  else if (ctrl >= 0x101 && ctrl <= 0x10F) { valid = i + (ctrl & 15) <= 15; src = l + (ctrl & 15); }
  else if (ctrl >= 0x111 && ctrl <= 0x11F) { valid = i - (ctrl & 15) >= 0; src = l - (ctrl & 15); }
  else src = dpp_src(l, ctrl);
  const int got = (int)(uint32_t)xchg((uint32_t)v, (enabled && valid) ? src : l);
  if (!enabled) return old;
  if (!valid) return bound_ctrl ? 0 : old;
  return got;
}
inline int readlane(int v, int l) { return (int)(uint32_t)xchg((uint32_t)v, l); }
template <typename T>
inline T shfl(T v, int src) {
  uint64_t b = 0;
  memcpy(&b, &v, sizeof(T));
  b = xchg(b, src);
  T r;
  memcpy(&r, &b, sizeof(T));
  return r;
}
inline unsigned long long ballot(bool p) {
  Wave& w = W();
  w.slot[lane()] = p ? 1 : 0;
  pthread_barrier_wait(&w.bar);
  unsigned long long m = 0;
  for (int i = 0; i < 64; ++i) m |= (unsigned long long)(w.slot[i] & 1) << i;
  pthread_barrier_wait(&w.bar);
  return m;
}
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
// v_mfma_f32_16x16x32_f16: A lane L = row L%16, k = 8*(L/16)+0..7; B lane L = col L%16, same k;
// D lane L = rows 4*(L/16)+i, col L%16.
inline f4 mfma(h8 a, h8 b, f4 c) {
  Wave& w = W();
  const int l = lane();
  for (int e = 0; e < 8; ++e) { w.ma[l][e] = a[e]; w.mb[l][e] = b[e]; }
  pthread_barrier_wait(&w.bar);
  f4 d = c;
  const int col = l & 15;
  for (int i = 0; i < 4; ++i) {
    const int row = 4 * (l >> 4) + i;
    double s = 0;
    for (int k = 0; k < 32; ++k) s += (double)(float)w.ma[row + 16 * (k >> 3)][k & 7] * (double)(float)w.mb[col + 16 * (k >> 3)][k & 7];
    d[i] = c[i] + (float)s;
  }
  pthread_barrier_wait(&w.bar);
  return d;
}
// v_mfma_f32_4x4x1_16B_f32: 16 blocks of 4 lanes; register i of lane L gets
// c[i] + a(lane 4*(L/4) + i) * b(lane L)
inline f4 mfma4x4x1(float a, float b, f4 c) {
  Wave& w = W();
  const int l = lane();
  uint32_t bits;
  memcpy(&bits, &a, 4);
  w.slot[l] = bits;
  pthread_barrier_wait(&w.bar);
  f4 d = c;
  for (int i = 0; i < 4; ++i) {
    const uint32_t ab = (uint32_t)w.slot[(l & ~3) + i];
    float av;
    memcpy(&av, &ab, 4);
    d[i] = fmaf(av, b, c[i]);
  }
  pthread_barrier_wait(&w.bar);
  return d;
}
extern unsigned char* dyn_lds;
// run a whole grid: one OS thread per lane, blocks one after the other
void launch_grid(dim3 grid, dim3 block, size_t lds, void (*fn)(void*), void* arg);
template <class F>
inline void launch(dim3 grid, dim3 block, size_t lds, F&& body) {
  launch_grid(grid, block, lds, [](void* p) { (*static_cast<F*>(p))(); }, &body);
}
}  // namespace simt

#define __builtin_amdgcn_update_dpp(old, src, ctrl, rm, bm, bc) simt::dpp_rows((old), (src), (ctrl), (rm), (bc))
#define __builtin_amdgcn_readlane(v, l) simt::readlane((v), (l))
#define __builtin_amdgcn_fence(...) ((void)0)
#define __builtin_amdgcn_wave_barrier() simt::wave_barrier()
#define __builtin_amdgcn_rsqf(x) (1.0f / sqrtf(x))
#define __builtin_amdgcn_rcpf(x) (1.0f / (x))
#define GEAR_ROWS_MIN_TOKENS 64   // the small emulated cases take the token-row kernels too
#define __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, x, y, z) \
  __builtin_bit_cast(gear::floatx4, simt::mfma(__builtin_bit_cast(simt::h8, (a)), __builtin_bit_cast(simt::h8, (b)), __builtin_bit_cast(simt::f4, (c))))
#define __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, c, x, y, z) \
  __builtin_bit_cast(gear::floatx4, simt::mfma4x4x1((a), (b), __builtin_bit_cast(simt::f4, (c))))
#define __syncthreads() pthread_barrier_wait(&simt::block_bar)
// shuffles inside segments of w lanes (w a power of two), as HIP defines them
template <typename T> inline T __shfl(T v, int src, int w = 64) { return simt::shfl(v, (simt::lane() & ~(w - 1)) + (src & (w - 1))); }
template <typename T> inline T __shfl_xor(T v, int m, int w = 64) {
  const int l = simt::lane(), t = l ^ m;
  return simt::shfl(v, (t & ~(w - 1)) == (l & ~(w - 1)) ? t : l);
}
template <typename T> inline T __shfl_up(T v, int o, int w = 64) {
  const int l = simt::lane();
  return simt::shfl(v, (l & (w - 1)) >= o ? l - o : l);
}
template <typename T> inline T __shfl_down(T v, int o, int w = 64) {
  const int l = simt::lane();
  return simt::shfl(v, (l & (w - 1)) + o < w ? l + o : l);
}
inline unsigned long long __ballot(bool p) { return simt::ballot(p); }
inline int __popcll(unsigned long long x) { return __builtin_popcountll(x); }
inline float __expf(float x) { return expf(x); }
inline float __int_as_float(int i) { float f; memcpy(&f, &i, 4); return f; }
inline int __float_as_int(float f) { int i; memcpy(&i, &f, 4); return i; }
inline float __uint_as_float(uint32_t i) { float f; memcpy(&f, &i, 4); return f; }
inline uint32_t __float_as_uint(float f) { uint32_t i; memcpy(&i, &f, 4); return i; }
inline float __fdiv_rn(float a, float b) { return a / b; }
inline float __fsub_rn(float a, float b) { return a - b; }
inline float __fmul_rn(float a, float b) { return a * b; }
inline int __popc(uint32_t x) { return __builtin_popcount(x); }
inline int __ffs(int x) { return __builtin_ffs(x); }
inline int __ffsll(long long x) { return __builtin_ffsll(x); }
inline int __clz(int x) { return x ? __builtin_clz((unsigned)x) : 32; }
inline int __clzll(long long x) { return x ? __builtin_clzll((unsigned long long)x) : 64; }
inline uint32_t atomicAdd(uint32_t* p, uint32_t v) { return __atomic_fetch_add(p, v, __ATOMIC_RELAXED); }
inline float atomicAdd(float* p, float v) {
  uint32_t* u = reinterpret_cast<uint32_t*>(p);
  uint32_t old = __atomic_load_n(u, __ATOMIC_RELAXED), nw;
  float f;
  do {
    memcpy(&f, &old, 4);
    const float g = f + v;
    memcpy(&nw, &g, 4);
  } while (!__atomic_compare_exchange_n(u, &old, nw, false, __ATOMIC_RELAXED, __ATOMIC_RELAXED));
  return f;
}
inline uint32_t atomicOr(uint32_t* p, uint32_t v) { return __atomic_fetch_or(p, v, __ATOMIC_RELAXED); }

#define hipLaunchKernelGGL(kernel, grid, block, lds, st, ...) simt::launch((grid), (block), (lds), [&] { kernel(__VA_ARGS__); })
