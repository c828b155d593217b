/*
 * gear.h -- C ABI of libgear: GEAR KV-cache compression (arXiv 2403.05527) and
 * the single-query attention read of the compressed cache, for AMD MI355X
 * (gfx950).  Plain C: pointers and sizes only, no C++ or torch types.
 *
 * Conventions (all entry points)
 *  - "device" pointers are HIP device memory of the current device, "host"
 *    pointers ordinary host memory.  Every buffer is allocated and freed by
 *    the caller; the library allocates nothing and keeps no global state.
 *  - Work is enqueued on the caller's hipStream_t (passed as void*, NULL = the
 *    default stream); no call synchronises with the host.  Inputs may be
 *    released once the stream has passed the call.
 *  - d_h (head dimension) must be 128.  Tensors are fp16, contiguous,
 *    [B, H, tokens, d_h] unless stated otherwise.  Inputs must be finite.
 *  - Return value: GEAR_OK (0) or a negative gear_status.  Arguments are
 *    validated on the host before anything is launched, so a failed call
 *    leaves the cache untouched.
 *  - A gear_cache is a small host-side descriptor owned by the caller.  It
 *    records what the device arena holds (segments, ranks, token counts) so
 *    that capacity and shape errors are caught without reading device memory.
 *    Calls on one gear_cache must be issued in stream order by one thread.
 */
#ifndef GEAR_H
#define GEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gear_status {
  GEAR_OK = 0,
  GEAR_EINVAL = -1,    /* bad / unsupported parameter, or NULL pointer            */
  GEAR_ECAPACITY = -2, /* arena, workspace, segment or chunk capacity exceeded     */
  GEAR_EALIGN = -3,    /* a pointer is not 16-byte aligned                         */
  GEAR_EHIP = -4       /* a HIP runtime call failed (launch error)                 */
} gear_status;

#define GEAR_MAX_CHUNKS 256
/* Size of the library's built-in scratch array (gear_decode_attn_static). */
#define GEAR_STATIC_SCRATCH_BYTES (32u << 20)

/* Hyper-parameters of Algorithm 1 of the paper plus the capacities of one
 * layer's cache. */
typedef struct gear_config {
  int32_t B;             /* batch                                                  */
  int32_t H_kv;          /* KV heads                                               */
  int32_t H_q;           /* query heads, multiple of H_kv, H_q/H_kv <= 8           */
  int32_t d_h;           /* head dimension, must be 128                            */
  int32_t bits;          /* b in {2, 4}  (Eq. 2)                                   */
  int32_t group;         /* g in {32, 64, 128}: Keys g tokens of one channel,      */
                         /* Values g channels of one token.  0: the coarse         */
                         /* per-vector grouping of the paper's background section  */
                         /* ("KCVT"): one group per Key channel over the tokens of */
                         /* a call, one per Value token over all H_kv*d_h channels */
  int32_t outlier_ppm;   /* s of Filter_s (Eq. 4) in parts per million of a        */
                         /* vector; 20000 = 2 %, 0 = GEAR-L (no sparse term)       */
  int32_t n_buf_cap;     /* n_b: streaming-buffer capacity, 1..255                 */
  int32_t n_prefill_max; /* capacity of the first (prefill) segment, <= 32768      */
  int32_t n_chunks_max;  /* number of flushed buffers that can be appended, <= 256 */
  int32_t rank_max;      /* largest rank any compress call will use, 0..8          */
  int32_t flags;         /* GEAR_FLAG_* bits, 0 = the method as the paper states it */
} gear_config;

/* Filter_s ranks each KV head's d_h channels of a Value token on their own (vector
 * length d_h, count ceil(s d_h) per head) instead of the token's row over all heads
 * (Eq. 4 read with X = V in R^{n x d}).  Every head is then independent of the others. */
#define GEAR_FLAG_V_FILTER_PER_HEAD 1

/* Host-side descriptor of one cache.  Filled by gear_cache_init, advanced by
 * gear_compress.  Treat the fields as read-only. */
typedef struct gear_cache {
  gear_config cfg;
  void*    arena;                        /* device                                 */
  uint64_t arena_bytes;
  int32_t  n_prefill;                    /* tokens in segment 0 (0 = none yet)     */
  int32_t  rank_prefill;
  int32_t  n_chunks;                     /* appended chunk segments                */
  int32_t  n_total;                      /* tokens in all segments                 */
  uint8_t  chunk_n[GEAR_MAX_CHUNKS];     /* tokens of chunk j                      */
  uint8_t  chunk_rank[GEAR_MAX_CHUNKS];  /* rank of chunk j                        */
} gear_cache;

/* Sizes the caller must provide for `cfg`: the device arena that holds the
 * compressed cache and a device workspace shared by gear_compress and
 * gear_decode_attn (scratch; contents need not survive between calls). */
int gear_cache_bytes(const gear_config* cfg, size_t* arena_bytes, size_t* workspace_bytes);

/* Binds a device arena (>= arena_bytes, 256-byte aligned) to `cache` (host,
 * out) and marks it empty.  Nothing is launched. */
int gear_cache_init(const gear_config* cfg, void* arena, size_t arena_bytes, gear_cache* cache);

/* Forgets every segment (the arena memory is reused). */
int gear_cache_reset(gear_cache* cache);

/*
 * Compress one segment of n tokens and append it (Algorithm 1: the prefill body
 * on the first call, the decoding-phase body on a flushed buffer afterwards):
 *   S = Filter_s(X)  (Eq. 4: per Key channel over the n tokens of this call,
 *                     per Value token over all H_kv*d_h channels; ties go to
 *                     the lower index),
 *   D = Quant_b(X - S) (Eq. 2 / Eq. 5, scale and zero-point stored in fp16),
 *   R = X - D - S, and per (batch, head) A, B = SVDSolver_rank(R) (Eq. 6,
 *   Algorithm 2 with `iters` rounds, start matrix init_B).
 * K, V      : device fp16 [B, H_kv, n, d_h].
 * n         : first call: 1..n_prefill_max; later calls: 1..n_buf_cap.
 * rank      : 0..rank_max (0 = no low-rank term); iters >= 1.
 * init_B    : device fp32 [2 (K,V), B, H_kv, d_h, rank], the start matrices B0 of
 *             Algorithm 2 (its random initialisation, taken as an input so that runs are
 *             reproducible), or NULL: the library then draws the same array on the
 *             device from `seed`: entry i (row-major) is ((z >> 40) - 2^23) / 2^23 with
 *             z = mix(seed + (i + 1) * 0x9E3779B97F4A7C15), mix(z): z ^= z >> 30,
 *             z *= 0xBF58476D1CE4E5B9, z ^= z >> 27, z *= 0x94D049BB133111EB,
 *             z ^= z >> 31 (64-bit arithmetic): uniform on a 24-bit grid in [-1, 1).
 * seed      : used only when init_B is NULL and rank > 0.
 * workspace : device, >= workspace_bytes of gear_cache_bytes.
 */
int gear_compress(gear_cache* cache, const void* K, const void* V, int32_t n, int32_t rank,
                  int32_t iters, const float* init_B, uint64_t seed, void* workspace,
                  size_t workspace_bytes, void* stream);

/*
 * gear_compress with the error-reduction (low-rank) term on the n_lowrank most recent tokens of
 * the call only: the ablation of Sec. 4.3 that recovers the quantization error of the p % most
 * recent prefill tokens (n_lowrank = ceil(p n / 100)).  SVDSolver runs on the residual rows of
 * those tokens; the earlier tokens get A = 0, i.e. Filter and Quant only.  n_lowrank = n is
 * gear_compress; n_lowrank = 0 stores the segment with rank 0.  (The other ablation of that
 * section, error reduction on the prefill tokens only -- "GEAR-L Prefill" --, needs no entry
 * point of its own: compress the flushed buffers with rank = 0.)
 */
int gear_compress_recent(gear_cache* cache, const void* K, const void* V, int32_t n, int32_t rank,
                         int32_t iters, const float* init_B, uint64_t seed, int32_t n_lowrank,
                         void* workspace, size_t workspace_bytes, void* stream);

/* X-hat = D + A B^T + S for every stored token (Algorithm 1, "replace X with
 * D + L + S"), rounded to fp16.  K_out, V_out: device fp16
 * [B, H_kv, n_total, d_h]; either may be NULL. */
int gear_decompress(const gear_cache* cache, void* K_out, void* V_out, void* stream);

/*
 * Single-query attention (Eq. 1) over the compressed cache followed by the
 * first n_buf rows of the fp16 streaming buffer, never materialising K-hat or
 * V-hat: softmax(q K^T / sqrt(d_h)) V per query head; query head i reads KV
 * head i / (H_q / H_kv).
 * q         : device fp16 [B, H_q, 1, d_h].
 * K_buf,V_buf: device fp16 [B, H_kv, n_buf_cap, d_h]; may be NULL when n_buf == 0.
 * n_buf     : 0..n_buf_cap; n_buf == 0 with an empty cache is GEAR_EINVAL.
 * out       : device fp16 [B, H_q, 1, d_h].
 * Value range: the products q[c] * scale_K(group, c) and p * scale_V (p <= 1) are fed to
 *             the matrix cores as fp16 numbers times at most 16, so finite outputs need
 *             |q[c] * scale_K| < 4094 and scale_V < 4094 for every entry (scale = (max - min)
 *             / (2^b - 1) of a group: K and V entries of magnitude up to ~1000 with |q| up to
 *             ~10 are inside).  Inputs beyond that are not detected: the outputs of the heads
 *             concerned are then inf or NaN and the call still returns GEAR_OK.
 */
int gear_decode_attn(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf,
                     int32_t n_buf, void* out, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * The same read for q_len query rows per head (chunked prefill, speculative decoding): the
 * packed codes are unpacked once and feed all rows' products.  The q_len newest tokens are the
 * last q_len of the n_buf buffer rows.  Every query attends to the whole compressed cache;
 * with causal != 0 query row j (0-based) attends to the buffer rows 0 .. n_buf - q_len + j
 * (Eq. 1 with the usual causal mask among the new tokens), otherwise to all n_buf rows.
 * q, out    : device fp16 [B, H_q, q_len, d_h].
 * q_len     : a power of two with q_len * (H_q / H_kv) <= 8 (longer blocks: several calls);
 *             causal needs n_buf >= q_len.  Otherwise GEAR_EINVAL.
 * workspace : the workspace of gear_cache_bytes; GEAR_ECAPACITY if the records of q_len rows do
 *             not fit behind those of one (they do whenever rank_max > 0).
 */
int gear_decode_attn_mq(const gear_cache* cache, const void* q, int32_t q_len, int32_t causal,
                        const void* K_buf, const void* V_buf, int32_t n_buf, void* out,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * gear_decode_attn for callers that cannot allocate device memory or bring a
 * workspace along: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same computation, same kernels and same results as
 * gear_decode_attn; the partial softmax records of the split blocks go to a
 * fixed array of GEAR_STATIC_SCRATCH_BYTES (32 MiB) that is part of the library
 * and that every GPU the library runs on holds until the process ends.  The call
 * allocates and frees nothing.
 *  - The records take B * H_q * (ceil(n_prefill / 512) + ceil(pieces / 4) + 1) * 520
 *    bytes (pieces = n_chunks, or 2 * n_chunks when n_buf_cap > 128); a cache
 *    that needs more than the array returns GEAR_ECAPACITY and launches nothing.
 *  - All calls on one GPU share that GPU's array: two calls that may overlap on
 *    one GPU (different streams, different threads) race and must be ordered
 *    by the caller.  Nothing has to be cleared between calls: every record a
 *    call reads it has written itself.
 */
int gear_decode_attn_static(const gear_cache* cache, const void* q, const void* K_buf, const void* V_buf,
                            int32_t n_buf, void* out, void* stream);

/*
 * Canonical views of the stored components (the physical arena layout is
 * private); used to check the library against an independent implementation.
 * which: 0 = Keys, 1 = Values.
 *  codes_u8 : device u8  [B, H_kv, n_total, d_h], one integer code per entry.
 *  scale/zero: device fp16; Keys [B, H_kv, NG, d_h] with NG = sum over segments
 *             of ceil(n_seg / g) (segments in append order); Values
 *             [B, H_kv, n_total, d_h / g].
 *  mask_u8  : device u8  [B, H_kv, n_total, d_h], 1 on the support of S.
 *  values   : device fp16 same shape, S itself (0 off the support).
 *  A_f16    : device fp16 [B, H_kv, n_seg, rank_seg]; B_f16: [B, H_kv, d_h, rank_seg].
 */
int gear_export_codes(const gear_cache* cache, int which, void* codes_u8, void* scale_f16,
                      void* zero_f16, void* stream);
int gear_export_sparse(const gear_cache* cache, int which, void* mask_u8, void* values_f16,
                       void* stream);
int gear_export_lowrank(const gear_cache* cache, int which, int seg, void* A_f16, void* B_f16,
                        void* stream);

/*
 * The sparse matrix S of Filter_s (Eq. 4) in the coordinate form the paper's Sec. 3.1
 * describes (index vectors plus one value vector), over all stored segments:
 *  nnz           : host, out.  Fixed by Eq. 4: every Key channel of a segment of n tokens
 *                  holds ceil(s n) entries, every Value token ceil(s H_kv d_h); the call
 *                  computes it on the host, so a first call with lin_index_i64 ==
 *                  value_f16 == NULL (nothing launched) tells the caller what to allocate.
 *  lin_index_i64 : device int64 [nnz], the linear index ((b * H_kv + h) * n_total + t) * d_h + c
 *                  of every entry, ascending (the two index vectors of the coordinate
 *                  form are index / d_h and index % d_h).
 *  value_f16     : device fp16 [nnz], the entries (bit copies of the input) in the same order.
 *  workspace     : device scratch, >= 4 * B * H_kv * n_total + 4 * ceil(B * H_kv * n_total / 1024)
 *                  + 512 bytes (the workspace of gear_cache_bytes is large enough whenever
 *                  n_total <= 8 * n_prefill_max); GEAR_ECAPACITY otherwise.
 */
int gear_export_sparse_coo(const gear_cache* cache, int which, int64_t* nnz, void* lin_index_i64,
                           void* value_f16, void* workspace, size_t workspace_bytes, void* stream);

const char* gear_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* GEAR_H */
