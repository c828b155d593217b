// C ABI of libgear: argument validation, arena / workspace layout and the launch
// sequences of the entry points declared in gear.h.
#include <string.h>
#include <mutex>

#include "gear_internal.h"
#include "gear_launch.h"

using namespace gear;

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

inline int outlier_count(long long n_v, long long ppm) {  // ceil(ppm * n_v / 1e6), clamped
  long long k = (ppm * n_v + 999999) / 1000000;
  if (k > n_v) k = n_v;
  if (k < 0) k = 0;
  return (int)k;
}

struct Region {  // byte offsets of one tensor's arrays inside a segment region
  size_t codes, sz, A, Bf, ell, table, pool, bytes;
  int n_cap, ng_cap, nblk_cap, ntile_cap;
  uint32_t pool_cap;
};

inline int group_of(const gear_config& c) { return c.group == 0 ? D : c.group; }   // tile-level group size
// outliers of one Value token over all heads
inline int v_outliers_per_token(const gear_config& c) {
  return (c.flags & GEAR_FLAG_V_FILTER_PER_HEAD) ? c.H_kv * outlier_count(D, c.outlier_ppm)
                                                 : outlier_count((long long)c.H_kv * D, c.outlier_ppm);
}

Region region_layout(const gear_config& c, bool is_k, int n_cap) {
  Region r;
  const size_t slabs = (size_t)c.B * c.H_kv;
  const int group = group_of(c);
  const int wpr = D * c.bits / 32, tpw = 32 / c.bits;
  n_cap = (n_cap + 7) & ~7;   // row strides of A, scale/zero and slots stay 16-byte aligned per slab
  r.n_cap = n_cap;
  r.ng_cap = (n_cap + group - 1) / group;
  r.nblk_cap = (n_cap + 4 * tpw - 1) / (4 * tpw);
  r.ntile_cap = (n_cap + TILE - 1) / TILE;
  size_t o = 0;
  r.codes = o;
  o += up(is_k ? slabs * n_cap * wpr * 4 : slabs * (size_t)r.nblk_cap * 2048);
  r.sz = o;
  o += up((is_k ? slabs * (size_t)r.ng_cap * D * 4 : slabs * (size_t)n_cap * (D / group) * 4) + 16);   // readers fetch whole 16-byte pieces
  r.A = o;
  o += up(slabs * (size_t)n_cap * (c.rank_max > 0 ? c.rank_max : 1) * 2 + 16);
  r.Bf = o;
  o += up(slabs * (size_t)D * (c.rank_max > 0 ? c.rank_max : 1) * 2);
  r.ell = o;
  o += up(is_k ? slabs * (size_t)n_cap * ELL_K * 4 : slabs * (size_t)r.ntile_cap * D * ELL_V * 4);
  r.table = o;
  o += up(slabs * (size_t)r.ntile_cap * 8);
  r.pool = o;
  if (is_k) {
    r.pool_cap = (uint32_t)D * outlier_count(n_cap, c.outlier_ppm);
    o += up(slabs * (size_t)r.pool_cap * 4);
  } else {
    r.pool_cap = (uint32_t)c.H_kv * r.ntile_cap * VPOOL_FIXED +   // reserved regions, then the worst case
                 (uint32_t)n_cap * v_outliers_per_token(c);
    o += up((size_t)c.B * r.pool_cap * 4);
  }
  r.bytes = o;
  return r;
}

struct ArenaLayout {
  Region kp, vp, kc, vc;   // prefill K/V, chunk K/V
  size_t off_kp, off_vp, off_chunks, chunk_stride, bytes;
};

ArenaLayout arena_layout(const gear_config& c) {
  ArenaLayout a;
  a.kp = region_layout(c, true, c.n_prefill_max);
  a.vp = region_layout(c, false, c.n_prefill_max);
  a.kc = region_layout(c, true, c.n_buf_cap);
  a.vc = region_layout(c, false, c.n_buf_cap);
  a.off_kp = 0;
  a.off_vp = a.kp.bytes;
  a.off_chunks = a.off_vp + a.vp.bytes;
  a.chunk_stride = a.kc.bytes + a.vc.bytes;
  a.bytes = a.off_chunks + a.chunk_stride * (size_t)c.n_chunks_max;
  return a;
}

struct WorkLayout {
  size_t thrK, thrV, vsz, pool_ctr, Bcur, partial, Atmp, cmat, dec, gram, resid, bytes;
  int gram_strips;
};

WorkLayout work_layout(const gear_config& c) {
  WorkLayout w;
  const size_t slabs = (size_t)c.B * c.H_kv;
  const int n_max = c.n_prefill_max > c.n_buf_cap ? c.n_prefill_max : c.n_buf_cap;
  const int npart = (n_max + 255) / 256;
  const int R = 8;
  size_t o = 0;
  w.thrK = o; o += up(slabs * D * sizeof(ThreshPair));
  w.thrV = o; o += up((size_t)c.B * n_max * sizeof(ThreshPair));
  w.vsz = o; o += up(c.group == 0 ? (size_t)c.B * n_max * 4 : 0);   // per-vector grouping: a Value token's (scale, zero)
  w.pool_ctr = o; o += up((slabs + (size_t)c.B) * 4);   // Key counters per slab, then Value counters per batch
  w.Bcur = o; o += up(slabs * D * R * 4);
  w.partial = o; o += up(slabs * (size_t)npart * (D * R + R * R) * 4);
  w.Atmp = o; o += up(slabs * (size_t)n_max * R * 4);
  w.cmat = o; o += up(slabs * R * R * 4);
  // decode records: one per 512 prefill tokens, one per four chunk pieces (a chunk is one
  // piece of up to 128 rows, two when n_buf_cap > 128), one for the buffer
  const int nsplit = (c.n_prefill_max + DECODE_SPLIT - 1) / DECODE_SPLIT;
  const int ncb = (c.n_chunks_max * (c.n_buf_cap > 128 ? 2 : 1) + 3) / 4;
  w.dec = o; o += up((size_t)c.B * c.H_q * (nsplit + ncb + 1) * DECODE_REC * 4);
  w.gram_strips = c.rank_max > 0 && n_max > 256 ? pi_gram_strips_max(n_max, (int)slabs) : 0;
  w.gram = o; o += up(slabs * (size_t)w.gram_strips * 36 * 256 * 4);
  // the filtered tensor for the low-rank passes; before it is written, the channel-major copy of the
  // keys of a long Key segment (see launch_k_select) lives in the same place
  w.resid = o;
  {
    const size_t resid = c.rank_max > 0 ? slabs * (size_t)n_max * D * 2 : 0;
    const size_t kt = c.n_prefill_max > 8192 ? slabs * (size_t)((c.n_prefill_max + 7) & ~7) * D * 2 : 0;
    o += up(resid > kt ? resid : kt);
  }
  w.bytes = o;
  return w;
}

bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

int check_config(const gear_config* c) {
  if (!c) return GEAR_EINVAL;
  if (c->B < 1 || c->H_kv < 1 || c->H_kv > 64 || c->H_q < c->H_kv || c->H_q % c->H_kv) return GEAR_EINVAL;
  const int gq = c->H_q / c->H_kv;
  if (!pow2(gq) || gq > 8) return GEAR_EINVAL;
  if (c->d_h != D) return GEAR_EINVAL;
  if (c->bits != 2 && c->bits != 4) return GEAR_EINVAL;
  if (c->group != 0 && c->group != 32 && c->group != 64 && c->group != 128) return GEAR_EINVAL;
  if (c->flags & ~GEAR_FLAG_V_FILTER_PER_HEAD) return GEAR_EINVAL;
  if (c->outlier_ppm < 0 || c->outlier_ppm > 500000) return GEAR_EINVAL;
  if (c->n_buf_cap < 1 || c->n_buf_cap > 255) return GEAR_EINVAL;
  if (c->n_prefill_max < 1 || c->n_prefill_max > 32768) return GEAR_EINVAL;
  if (c->n_chunks_max < 0 || c->n_chunks_max > GEAR_MAX_CHUNKS) return GEAR_EINVAL;
  if (c->rank_max < 0 || c->rank_max > 8) return GEAR_EINVAL;
  if ((long long)c->B * c->H_kv > 65535) return GEAR_EINVAL;  // grid.y
  return GEAR_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Dims make_dims(const gear_config& c) {
  Dims d;
  d.B = c.B; d.H = c.H_kv; d.Hq = c.H_q;
  d.bits = c.bits; d.g = group_of(c); d.ppm = c.outlier_ppm;
  d.kcvt = c.group == 0 ? 1 : 0;
  d.vhead = (c.flags & GEAR_FLAG_V_FILTER_PER_HEAD) ? 1 : 0;
  d.wpr = D * c.bits / 32;
  d.tpw = 32 / c.bits;
  d.qmax = (float)((1 << c.bits) - 1);
  return d;
}

SegView make_view(char* base, const Region& r, int n, int rank, int t0, int g0) {
  SegView v;
  v.codes = reinterpret_cast<uint32_t*>(base + r.codes);
  v.sz = reinterpret_cast<uint32_t*>(base + r.sz);
  v.A = reinterpret_cast<uint16_t*>(base + r.A);
  v.Bf = reinterpret_cast<uint16_t*>(base + r.Bf);
  v.ell = reinterpret_cast<uint32_t*>(base + r.ell);
  v.sp_table = reinterpret_cast<uint2*>(base + r.table);
  v.sp_pool = reinterpret_cast<uint32_t*>(base + r.pool);
  v.n = n; v.n_cap = r.n_cap; v.rank = rank;
  v.ng_cap = r.ng_cap; v.nblk_cap = r.nblk_cap; v.ntile_cap = r.ntile_cap;
  v.pool_cap = r.pool_cap;
  v.t0 = t0; v.g0 = g0;
  return v;
}

// seg 0 = prefill, seg j >= 1 = chunk j-1
void seg_views(const gear_cache* cache, const ArenaLayout& a, int seg, int n, int rank, SegView* k, SegView* v) {
  char* base = static_cast<char*>(cache->arena);
  const int g = cache->cfg.group == 0 ? 1 << 30 : cache->cfg.group;   // per-vector grouping: one Key group per segment
  if (seg == 0) {
    *k = make_view(base + a.off_kp, a.kp, n, rank, 0, 0);
    *v = make_view(base + a.off_vp, a.vp, n, rank, 0, 0);
    return;
  }
  int t0 = cache->n_prefill, g0 = (cache->n_prefill + g - 1) / g;
  for (int j = 0; j < seg - 1; ++j) {
    t0 += cache->chunk_n[j];
    g0 += (cache->chunk_n[j] + g - 1) / g;
  }
  char* cb = base + a.off_chunks + a.chunk_stride * (size_t)(seg - 1);
  *k = make_view(cb, a.kc, n, rank, t0, g0);
  *v = make_view(cb + a.kc.bytes, a.vc, n, rank, t0, g0);
}

int n_segments(const gear_cache* c) { return (c->n_prefill > 0 ? 1 : 0) + c->n_chunks; }
int seg_n(const gear_cache* c, int seg) { return seg == 0 ? c->n_prefill : c->chunk_n[seg - 1]; }
int seg_rank(const gear_cache* c, int seg) { return seg == 0 ? c->rank_prefill : c->chunk_rank[seg - 1]; }
int total_groups(const gear_cache* c) {
  const int g = c->cfg.group == 0 ? 1 << 30 : c->cfg.group;
  int ng = (c->n_prefill + g - 1) / g;
  for (int j = 0; j < c->n_chunks; ++j) ng += (c->chunk_n[j] + g - 1) / g;
  return ng;
}

int check_cache(const gear_cache* c) {
  if (!c || !c->arena) return GEAR_EINVAL;
  return check_config(&c->cfg);
}

#define GEAR_HIP(expr)                           \
  do {                                           \
    hipError_t e__ = (expr);                     \
    if (e__ != hipSuccess) return GEAR_EHIP;     \
  } while (0)


// ---------------------------------------------------------------------------
// Scratch memory of gear_decode_attn_static: a fixed array in device memory that
// every GPU holds from the moment the library is loaded until the process ends.
// In host code the array's name is only a handle; the address the kernels get is
// looked up once per device with hipGetSymbolAddress and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[GEAR_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_ptr[MAX_DEVICES];   // per device: address of that device's copy of `scratch`, nullptr until looked up

// Address of the current device's scratch array (looked up on the first call on that device).
int current_device_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return GEAR_EHIP;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GEAR_EHIP;
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return GEAR_OK;
}

// Common body of the two decode entry points.  `partial` holds the split records
// (at least decode_record_bytes(cache) bytes).
size_t decode_record_bytes(const gear_cache* cache) {
  const gear_config& c = cache->cfg;
  const int nsplit = (cache->n_prefill + DECODE_SPLIT - 1) / DECODE_SPLIT;
  const int ncb = (cache->n_chunks * (c.n_buf_cap > 128 ? 2 : 1) + 3) / 4;
  return (size_t)c.B * c.H_q * (nsplit + ncb + 1) * DECODE_REC * 4;
}

int decode_checked(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf, int32_t n_buf,
                   int q_len, int causal, void* out, float* partial, void* stream) {
  const gear_config& c = cache->cfg;
  const ArenaLayout a = arena_layout(c);
  const Dims dm = make_dims(c);
  SegView k0, v0;
  seg_views(cache, a, 0, cache->n_prefill, cache->rank_prefill, &k0, &v0);
  ChunkSet cs;
  memset(&cs, 0, sizeof(cs));
  {
    // views of chunk 0 (token offsets are irrelevant for attention)
    char* cb = static_cast<char*>(cache->arena) + a.off_chunks;
    cs.k0 = make_view(cb, a.kc, 0, 0, 0, 0);
    cs.v0 = make_view(cb + a.kc.bytes, a.vc, 0, 0, 0, 0);
  }
  cs.stride = a.chunk_stride;
  cs.n_chunks = cache->n_chunks;
  for (int j = 0; j < cache->n_chunks; ++j) {
    cs.n[j] = cache->chunk_n[j];
    cs.rank[j] = cache->chunk_rank[j];
  }
  GEAR_HIP(launch_decode(dm, k0, v0, cs, static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(K_buf),
                         static_cast<const uint16_t*>(V_buf), n_buf, c.n_buf_cap, c.rank_max, q_len, causal,
                         static_cast<uint16_t*>(out), partial, static_cast<hipStream_t>(stream)));
  return GEAR_OK;
}

int check_decode_args(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf, int32_t n_buf,
                      const void* out) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  const gear_config& c = cache->cfg;
  if (!q || !out) return GEAR_EINVAL;
  if (n_buf < 0 || n_buf > c.n_buf_cap) return GEAR_EINVAL;
  if (n_buf > 0 && (!K_buf || !V_buf)) return GEAR_EINVAL;
  if (n_buf == 0 && cache->n_total == 0) return GEAR_EINVAL;
  if (!aligned16(q) || !aligned16(out) || (K_buf && !aligned16(K_buf)) || (V_buf && !aligned16(V_buf))) return GEAR_EALIGN;
  return GEAR_OK;
}

}  // namespace

extern "C" {

int gear_cache_bytes(const gear_config* cfg, size_t* arena_bytes, size_t* workspace_bytes) {
  const int rc = check_config(cfg);
  if (rc) return rc;
  if (arena_bytes) *arena_bytes = arena_layout(*cfg).bytes;
  if (workspace_bytes) *workspace_bytes = work_layout(*cfg).bytes;
  return GEAR_OK;
}

int gear_cache_init(const gear_config* cfg, void* arena, size_t arena_bytes, gear_cache* cache) {
  const int rc = check_config(cfg);
  if (rc) return rc;
  if (!arena || !cache) return GEAR_EINVAL;
  if (reinterpret_cast<uintptr_t>(arena) & (ALIGN - 1)) return GEAR_EALIGN;
  if (arena_bytes < arena_layout(*cfg).bytes) return GEAR_ECAPACITY;
  memset(cache, 0, sizeof(*cache));
  cache->cfg = *cfg;
  cache->arena = arena;
  cache->arena_bytes = arena_bytes;
  return GEAR_OK;
}

int gear_cache_reset(gear_cache* cache) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  cache->n_prefill = cache->rank_prefill = cache->n_chunks = cache->n_total = 0;
  return GEAR_OK;
}

int gear_compress_recent(gear_cache* cache, const void* K, const void* V, int32_t n, int32_t rank, int32_t iters,
                         const float* init_B, uint64_t seed, int32_t n_lowrank, void* workspace, size_t workspace_bytes,
                         void* stream) {
  int rc = check_cache(cache);
  if (rc) return rc;
  const gear_config& c = cache->cfg;
  if (!K || !V || !workspace) return GEAR_EINVAL;
  if (n < 1 || rank < 0 || rank > c.rank_max || iters < 1 || iters > 64) return GEAR_EINVAL;
  if (n_lowrank < 0 || n_lowrank > n) return GEAR_EINVAL;
  if (n_lowrank == 0) rank = 0;          // no token takes the low-rank term
  const int t_lr = n - n_lowrank;
  if (!aligned16(K) || !aligned16(V) || !aligned16(workspace) || (init_B && !aligned16(init_B))) return GEAR_EALIGN;
  const bool first = cache->n_prefill == 0;
  if (first) {
    if (n > c.n_prefill_max) return GEAR_ECAPACITY;
  } else {
    if (n > c.n_buf_cap) return GEAR_ECAPACITY;
    if (cache->n_chunks >= c.n_chunks_max) return GEAR_ECAPACITY;
  }
  const WorkLayout w = work_layout(c);
  if (workspace_bytes < w.bytes) return GEAR_ECAPACITY;

  const ArenaLayout a = arena_layout(c);
  const Dims dm = make_dims(c);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const int seg = first ? 0 : cache->n_chunks + 1;
  SegView ks, vs;
  seg_views(cache, a, seg, n, rank, &ks, &vs);
  const uint16_t* Kp = static_cast<const uint16_t*>(K);
  const uint16_t* Vp = static_cast<const uint16_t*>(V);
  ThreshPair* thrK = reinterpret_cast<ThreshPair*>(ws + w.thrK);
  ThreshPair* thrV = reinterpret_cast<ThreshPair*>(ws + w.thrV);
  uint32_t* pool_ctr = reinterpret_cast<uint32_t*>(ws + w.pool_ctr);

  const int kv_k = outlier_count(n, c.outlier_ppm);
  const bool vhead = (c.flags & GEAR_FLAG_V_FILTER_PER_HEAD) != 0;
  const int kv_v = outlier_count(vhead ? D : (long long)c.H_kv * D, c.outlier_ppm);   // per Value vector
  // the Key selection kernel also finds a channel's (scale, zero) under the per-vector grouping
  if (c.outlier_ppm > 0 || dm.kcvt) {
    GEAR_HIP(launch_k_select(Kp, dm, n, (kv_k + 1) / 2, kv_k / 2, thrK, pool_ctr, c.B * c.H_kv + c.B, ks,
                             n > 8192 ? reinterpret_cast<uint16_t*>(ws + w.resid) : nullptr, st));
  }
  // Keys: quantize (leaving Y = X - S in the workspace), then their power iteration;
  // Values reuse the same buffer afterwards.
  uint16_t* resid = rank > 0 ? reinterpret_cast<uint16_t*>(ws + w.resid) : nullptr;
  float* Bcur = reinterpret_cast<float*>(ws + w.Bcur);
  float* partial = reinterpret_cast<float*>(ws + w.partial);
  float* Atmp = reinterpret_cast<float*>(ws + w.Atmp);
  float* cmat = reinterpret_cast<float*>(ws + w.cmat);
  float* gram = reinterpret_cast<float*>(ws + w.gram);
  uint32_t* vsz = reinterpret_cast<uint32_t*>(ws + w.vsz);
  GEAR_HIP(launch_k_quant(Kp, ks, dm, n, thrK, pool_ctr, resid, st));
  if (rank > 0) GEAR_HIP(launch_power_iteration(true, resid, ks, dm, n, t_lr, iters, init_B, seed, Bcur, partial, Atmp, cmat, gram, w.gram_strips, st));
  GEAR_HIP(launch_v_filter_quant(Vp, vs, dm, n, (kv_v + 1) / 2, kv_v / 2, thrV, vsz, pool_ctr + (size_t)c.B * c.H_kv, resid, st));
  if (rank > 0)
    GEAR_HIP(launch_power_iteration(false, resid, vs, dm, n, t_lr, iters, init_B, seed, Bcur, partial, Atmp, cmat, gram, w.gram_strips, st));

  if (first) {
    cache->n_prefill = n;
    cache->rank_prefill = rank;
  } else {
    cache->chunk_n[cache->n_chunks] = (uint8_t)n;
    cache->chunk_rank[cache->n_chunks] = (uint8_t)rank;
    cache->n_chunks += 1;
  }
  cache->n_total += n;
  return GEAR_OK;
}

int gear_compress(gear_cache* cache, const void* K, const void* V, int32_t n, int32_t rank, int32_t iters,
                  const float* init_B, uint64_t seed, void* workspace, size_t workspace_bytes, void* stream) {
  return gear_compress_recent(cache, K, V, n, rank, iters, init_B, seed, n, workspace, workspace_bytes, stream);
}

int gear_decompress(const gear_cache* cache, void* K_out, void* V_out, void* stream) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  if (!K_out && !V_out) return GEAR_EINVAL;
  if ((K_out && !aligned16(K_out)) || (V_out && !aligned16(V_out))) return GEAR_EALIGN;
  const ArenaLayout a = arena_layout(cache->cfg);
  const Dims dm = make_dims(cache->cfg);
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int seg = 0; seg <= cache->n_chunks; ++seg) {
    if (seg == 0 && cache->n_prefill == 0) continue;
    SegView ks, vs;
    seg_views(cache, a, seg, seg_n(cache, seg), seg_rank(cache, seg), &ks, &vs);
    GEAR_HIP(launch_decompress(dm, ks, vs, static_cast<uint16_t*>(K_out), static_cast<uint16_t*>(V_out),
                               cache->n_total, st));
  }
  return GEAR_OK;
}

int gear_decode_attn(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf, int32_t n_buf,
                     void* out, void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_decode_args(cache, q, K_buf, V_buf, n_buf, out);
  if (rc) return rc;
  if (!workspace) return GEAR_EINVAL;
  if (!aligned16(workspace)) return GEAR_EALIGN;
  const WorkLayout w = work_layout(cache->cfg);
  if (workspace_bytes < w.bytes) return GEAR_ECAPACITY;
  return decode_checked(cache, q, K_buf, V_buf, n_buf, 1, 0, out,
                        reinterpret_cast<float*>(static_cast<char*>(workspace) + w.dec), stream);
}

int gear_decode_attn_mq(const gear_cache* cache, const void* q, int32_t q_len, int32_t causal, const void* K_buf,
                        const void* V_buf, int32_t n_buf, void* out, void* workspace, size_t workspace_bytes,
                        void* stream) {
  const int rc = check_decode_args(cache, q, K_buf, V_buf, n_buf, out);
  if (rc) return rc;
  const gear_config& c = cache->cfg;
  if (q_len < 1 || !pow2(q_len) || q_len * (c.H_q / c.H_kv) > 8) return GEAR_EINVAL;
  if (causal && n_buf < q_len) return GEAR_EINVAL;   // the q_len newest tokens are buffer rows
  if (!workspace) return GEAR_EINVAL;
  if (!aligned16(workspace)) return GEAR_EALIGN;
  const WorkLayout w = work_layout(c);
  // the records of all q_len rows; what follows them in the workspace is scratch of gear_compress
  if (workspace_bytes < w.bytes || w.dec + decode_record_bytes(cache) * (size_t)q_len > w.bytes) return GEAR_ECAPACITY;
  return decode_checked(cache, q, K_buf, V_buf, n_buf, q_len, causal ? 1 : 0, out,
                        reinterpret_cast<float*>(static_cast<char*>(workspace) + w.dec), stream);
}

int gear_decode_attn_static(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf,
                            int32_t n_buf, void* out, void* stream) {
  const int rc = check_decode_args(cache, q, K_buf, V_buf, n_buf, out);
  if (rc) return rc;
  if (decode_record_bytes(cache) > (size_t)GEAR_STATIC_SCRATCH_BYTES) return GEAR_ECAPACITY;
  void* sp = nullptr;
  const int rs = current_device_scratch(&sp);
  if (rs) return rs;
  return decode_checked(cache, q, K_buf, V_buf, n_buf, 1, 0, out, static_cast<float*>(sp), stream);
}

int gear_export_codes(const gear_cache* cache, int which, void* codes_u8, void* scale_f16, void* zero_f16,
                      void* stream) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  if ((which != 0 && which != 1) || !codes_u8 || !scale_f16 || !zero_f16) return GEAR_EINVAL;
  const ArenaLayout a = arena_layout(cache->cfg);
  const Dims dm = make_dims(cache->cfg);
  const int ng_total = total_groups(cache);
  for (int seg = 0; seg <= cache->n_chunks; ++seg) {
    if (seg == 0 && cache->n_prefill == 0) continue;
    SegView ks, vs;
    seg_views(cache, a, seg, seg_n(cache, seg), seg_rank(cache, seg), &ks, &vs);
    GEAR_HIP(launch_export_codes(dm, which == 0 ? ks : vs, which == 0, static_cast<uint8_t*>(codes_u8),
                                 static_cast<uint16_t*>(scale_f16), static_cast<uint16_t*>(zero_f16),
                                 cache->n_total, ng_total, static_cast<hipStream_t>(stream)));
  }
  return GEAR_OK;
}

int gear_export_sparse(const gear_cache* cache, int which, void* mask_u8, void* values_f16, void* stream) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  if ((which != 0 && which != 1) || !mask_u8 || !values_f16) return GEAR_EINVAL;
  if (!aligned16(mask_u8) || !aligned16(values_f16)) return GEAR_EALIGN;
  const ArenaLayout a = arena_layout(cache->cfg);
  const Dims dm = make_dims(cache->cfg);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t entries = (size_t)cache->cfg.B * cache->cfg.H_kv * cache->n_total * D;
  GEAR_HIP(launch_fill_u32(static_cast<uint32_t*>(mask_u8), 0u, entries / 4, st));
  GEAR_HIP(launch_fill_u32(static_cast<uint32_t*>(values_f16), 0u, entries / 2, st));
  for (int seg = 0; seg <= cache->n_chunks; ++seg) {
    if (seg == 0 && cache->n_prefill == 0) continue;
    SegView ks, vs;
    seg_views(cache, a, seg, seg_n(cache, seg), seg_rank(cache, seg), &ks, &vs);
    GEAR_HIP(launch_export_sparse(dm, which == 0 ? ks : vs, which == 0, static_cast<uint8_t*>(mask_u8),
                                  static_cast<uint16_t*>(values_f16), cache->n_total, st));
  }
  return GEAR_OK;
}

int gear_export_sparse_coo(const gear_cache* cache, int which, int64_t* nnz, void* lin_index_i64, void* value_f16,
                           void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  if ((which != 0 && which != 1) || !nnz) return GEAR_EINVAL;
  const gear_config& c = cache->cfg;
  // the counts are fixed by Filter_s: per Key channel of a segment, per Value token
  long long total = 0;
  for (int seg = 0; seg <= cache->n_chunks; ++seg) {
    if (seg == 0 && cache->n_prefill == 0) continue;
    const long long n = seg_n(cache, seg);
    total += which == 0 ? (long long)c.B * c.H_kv * D * outlier_count(n, c.outlier_ppm)
                        : (long long)c.B * n * v_outliers_per_token(c);
  }
  *nnz = total;
  if (!lin_index_i64 && !value_f16) return GEAR_OK;   // size query
  if (!lin_index_i64 || !value_f16 || !workspace) return GEAR_EINVAL;
  if (!aligned16(lin_index_i64) || !aligned16(value_f16) || !aligned16(workspace)) return GEAR_EALIGN;
  if (total == 0) return GEAR_OK;
  if (total >= (1ll << 32)) return GEAR_ECAPACITY;
  const size_t rows = (size_t)c.B * c.H_kv * cache->n_total;
  const size_t need = up(rows * 4) + up(((rows + 1023) / 1024) * 4);
  if (workspace_bytes < need) return GEAR_ECAPACITY;
  uint32_t* rowcnt = static_cast<uint32_t*>(workspace);
  uint32_t* sums = reinterpret_cast<uint32_t*>(static_cast<char*>(workspace) + up(rows * 4));
  const ArenaLayout a = arena_layout(c);
  const Dims dm = make_dims(c);
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int pass = 0; pass < 2; ++pass) {
    for (int seg = 0; seg <= cache->n_chunks; ++seg) {
      if (seg == 0 && cache->n_prefill == 0) continue;
      SegView ks, vs;
      seg_views(cache, a, seg, seg_n(cache, seg), seg_rank(cache, seg), &ks, &vs);
      GEAR_HIP(launch_coo_tiles(dm, which == 0 ? ks : vs, which == 0, pass == 0, rowcnt, static_cast<long long*>(lin_index_i64),
                                static_cast<uint16_t*>(value_f16), cache->n_total, st));
    }
    if (pass == 0) GEAR_HIP(launch_exclusive_scan(rowcnt, rows, sums, st));
  }
  return GEAR_OK;
}

int gear_export_lowrank(const gear_cache* cache, int which, int seg, void* A_f16, void* B_f16, void* stream) {
  const int rc = check_cache(cache);
  if (rc) return rc;
  if ((which != 0 && which != 1) || !A_f16 || !B_f16) return GEAR_EINVAL;
  if (seg < 0 || seg > cache->n_chunks || (seg == 0 && cache->n_prefill == 0)) return GEAR_EINVAL;
  const ArenaLayout a = arena_layout(cache->cfg);
  const Dims dm = make_dims(cache->cfg);
  SegView ks, vs;
  seg_views(cache, a, seg, seg_n(cache, seg), seg_rank(cache, seg), &ks, &vs);
  GEAR_HIP(launch_export_lowrank(dm, which == 0 ? ks : vs, static_cast<uint16_t*>(A_f16),
                                 static_cast<uint16_t*>(B_f16), static_cast<hipStream_t>(stream)));
  return GEAR_OK;
}

const char* gear_strerror(int status) {
  switch (status) {
    case GEAR_OK: return "ok";
    case GEAR_EINVAL: return "invalid or unsupported argument";
    case GEAR_ECAPACITY: return "capacity exceeded (arena, workspace, segment or chunk count)";
    case GEAR_EALIGN: return "pointer not sufficiently aligned";
    case GEAR_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

}  // extern "C"
