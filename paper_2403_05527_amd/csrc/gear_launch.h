// Host-side launch functions of the kernel translation units.
#pragma once
#include "gear_internal.h"

namespace gear {

// Chunk segments live in equally sized regions; view j = view 0 advanced by
// j * stride bytes on every pointer.
struct ChunkSet {
  SegView k0, v0;       // views of chunk 0 (n / rank filled per chunk on the device)
  uint64_t stride;      // bytes between consecutive chunk regions
  int n_chunks;
  uint8_t n[GEAR_MAX_CHUNKS];
  uint8_t rank[GEAR_MAX_CHUNKS];
};

hipError_t launch_fill_u32(uint32_t* p, uint32_t v, size_t count, hipStream_t st);

// also clears zero[0 .. zero_count) (the list counters of the call); under the per-vector grouping it also writes
// every channel's (scale, zero) of the segment sv
hipError_t launch_k_select(const uint16_t* K, const Dims& dm, int n, int k_top, int k_bot, ThreshPair* thrK,
                           uint32_t* zero, int zero_count, const SegView& sv, uint16_t* kt_scratch, hipStream_t st);
// Yout (nullable): [slab][n][128] fp16, Y = X - S (the input with its outliers zeroed), from
// which the power iteration re-derives the residual R = Y - D-hat.
hipError_t launch_k_quant(const uint16_t* K, const SegView& sv, const Dims& dm, int n, const ThreshPair* thrK,
                          uint32_t* pool_ctr, uint16_t* Yout, hipStream_t st);
// k_top / k_bot: per Value vector (the token's row over all heads, or one head's channels of it); vsz: [B][n] words,
// a token's (scale, zero) under the per-vector grouping
hipError_t launch_v_filter_quant(const uint16_t* V, const SegView& sv, const Dims& dm, int n, int k_top,
                                 int k_bot, ThreshPair* thrV, uint32_t* vsz, uint32_t* pool_ctr, uint16_t* Yout,
                                 hipStream_t st);

int pi_padded_rank(int rank);
// gram: [slab][strip][36 * 256] floats, the partial Gram matrices of the residual (segments of more than 256 tokens
// with iters > 1); gram_strips_cap: strips per slab it has room for (pi_gram_strips_max of the largest segment)
int pi_gram_strips_max(int n_max, int slabs);
// init_B: the whole start array [2 (K, V), B, H, 128, rank] (the launcher takes this tensor's half), or
// nullptr: the same array is drawn from `seed` (start_entry in gear_internal.h)
// t_lr: first token of the segment that takes part in the low-rank term (rows before it get A = 0)
hipError_t launch_power_iteration(bool is_k, const uint16_t* Yf, const SegView& sv, const Dims& dm, int n, int t_lr, int iters,
                                  const float* init_B, uint64_t seed, float* Bcur, float* partial, float* Atmp, float* cmat,
                                  float* gram, int gram_strips_cap, hipStream_t st);

constexpr int DECODE_TS = 256;           // rows per pass of the chunk / buffer path
constexpr int DECODE_SPLIT = 512;        // prefill tokens per split block
constexpr int DECODE_REC = 2 + D;        // floats per partial record: m, l, o[128]
// q: [B, H_q, q_len, 128]; q_len a power of two with (H_q / H) * q_len <= 8; causal: query row j sees the buffer
// rows 0 .. n_buf - q_len + j; partial: B * H_q * q_len * (records per row) * DECODE_REC floats
hipError_t launch_decode(const Dims& dm, const SegView& k0, const SegView& v0, const ChunkSet& cs,
                         const uint16_t* q, const uint16_t* Kbuf, const uint16_t* Vbuf, int n_buf,
                         int n_buf_cap, int rank_cap, int q_len, int causal, uint16_t* out, float* partial,
                         hipStream_t st);

hipError_t launch_decompress(const Dims& dm, const SegView& ks, const SegView& vs, uint16_t* Kout,
                             uint16_t* Vout, int n_total, hipStream_t st);
hipError_t launch_export_codes(const Dims& dm, const SegView& sv, bool is_k, uint8_t* codes, uint16_t* scale,
                               uint16_t* zero, int n_total, int ng_total, hipStream_t st);
hipError_t launch_export_sparse(const Dims& dm, const SegView& sv, bool is_k, uint8_t* mask, uint16_t* vals,
                                int n_total, hipStream_t st);
// COO view of S: count = true writes every token row's outlier count to rowcnt[slab * n_total + t]; count = false
// writes the rows' entries from the positions rowcnt then holds (launch_exclusive_scan in between; sums: scratch of
// ceil(count / 1024) words)
hipError_t launch_coo_tiles(const Dims& dm, const SegView& sv, bool is_k, bool count, uint32_t* rowcnt, long long* lin,
                            uint16_t* vals, int n_total, hipStream_t st);
hipError_t launch_exclusive_scan(uint32_t* v, size_t count, uint32_t* sums, hipStream_t st);
hipError_t launch_export_lowrank(const Dims& dm, const SegView& sv, uint16_t* A, uint16_t* Bf, hipStream_t st);

}  // namespace gear
