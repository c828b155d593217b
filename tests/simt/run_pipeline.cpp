// Runs the library's C ABI end to end on the CPU emulation: prefill compress, chunk compresses,
// decode attention (one and two query rows), decompress, the canonical views.  Inputs and outputs are raw files in the directory given as argv[1]
// (written and read by tests/test_cpu_emulation.py).
// Plain C I/O only, so a memory-sanitizer build sees no uninstrumented C++ library code.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "gear.h"
static void* rd(const char* dir, const char* name, int idx) {
  char p[512];
  if (idx >= 0) snprintf(p, sizeof p, "%s/%s%d.bin", dir, name, idx); else snprintf(p, sizeof p, "%s/%s.bin", dir, name);
  FILE* f = fopen(p, "rb"); if (!f) { perror(p); exit(1); }
  fseek(f, 0, SEEK_END); long n = ftell(f); fseek(f, 0, SEEK_SET);
  void* v = aligned_alloc(256, (n + 255) / 256 * 256 + 256);
  if (n && fread(v, 1, n, f) != (size_t)n) exit(1);
  fclose(f); return v;
}
static void wr(const char* dir, const char* name, const void* v, size_t bytes) {
  char p[512]; snprintf(p, sizeof p, "%s/%s.bin", dir, name);
  FILE* f = fopen(p, "wb"); fwrite(v, 1, bytes, f); fclose(f);
}
#define CK(x) do { int s_ = (x); if (s_ != GEAR_OK) { fprintf(stderr, "%s -> %s\n", #x, gear_strerror(s_)); return 3; } } while (0)
int main(int argc, char** argv) {
  const char* dir = argv[1];
  int B, H, Hq, bits, g, ppm, n, rank, nchunks, chunk_n, rank_chunk, n_buf, n_buf_cap, iters, flags = 0, n_lowrank = -1;
  char p[512]; snprintf(p, sizeof p, "%s/meta.txt", dir);
  FILE* f = fopen(p, "r");
  if (fscanf(f, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d %d", &B, &H, &Hq, &bits, &g, &ppm, &n, &rank, &nchunks, &chunk_n, &rank_chunk, &n_buf, &n_buf_cap, &iters, &flags, &n_lowrank) < 14) return 1;
  fclose(f);
  gear_config cfg{B, H, Hq, 128, bits, g, ppm, n_buf_cap, n, nchunks > 0 ? nchunks : 1, rank > rank_chunk ? rank : rank_chunk, flags};
  size_t ab = 0, wb = 0;
  CK(gear_cache_bytes(&cfg, &ab, &wb));
  void* arena = aligned_alloc(256, (ab + 255) / 256 * 256);
  void* work = aligned_alloc(256, (wb + 255) / 256 * 256);
#ifndef EMU_NO_FILL
  memset(arena, 0xEE, ab); memset(work, 0xEE, wb);
#endif
  gear_cache cache;
  CK(gear_cache_init(&cfg, arena, ab, &cache));
  void *K = rd(dir, "K", -1), *V = rd(dir, "V", -1), *ib = rd(dir, "ib", -1);
  fprintf(stderr, "compress prefill n=%d\n", n);
  if (n_lowrank >= 0)   // the low-rank term on the most recent n_lowrank tokens of the call only
    CK(gear_compress_recent(&cache, K, V, n, rank, iters, rank ? (const float*)ib : nullptr, 0, n_lowrank, work, wb, nullptr));
  else
    CK(gear_compress(&cache, K, V, n, rank, iters, rank ? (const float*)ib : nullptr, 0, work, wb, nullptr));
  for (int j = 0; j < nchunks; ++j) {
    void *Kc = rd(dir, "Kc", j), *Vc = rd(dir, "Vc", j), *ibc = rd(dir, "ibc", j);
    fprintf(stderr, "compress chunk %d n=%d\n", j, chunk_n);
    CK(gear_compress(&cache, Kc, Vc, chunk_n, rank_chunk, iters, (const float*)ibc, 0, work, wb, nullptr));
  }
  void *q = rd(dir, "q", -1), *Kb = rd(dir, "Kb", -1), *Vb = rd(dir, "Vb", -1);
  const size_t ob = (size_t)B * Hq * 128 * 2;
  void* out = aligned_alloc(256, (ob + 255) / 256 * 256);
  fprintf(stderr, "decode n_buf=%d\n", n_buf);
  CK(gear_decode_attn(&cache, q, Kb, Vb, n_buf, out, work, wb, nullptr));
  wr(dir, "out", out, ob);
  const size_t ntot = (size_t)cache.n_total, hb = (size_t)B * H * ntot * 128 * 2;
  void *Kh = aligned_alloc(256, (hb + 255) / 256 * 256), *Vh = aligned_alloc(256, (hb + 255) / 256 * 256);
  fprintf(stderr, "decompress n_total=%zu\n", ntot);
  CK(gear_decompress(&cache, Kh, Vh, nullptr));
  wr(dir, "Khat", Kh, hb); wr(dir, "Vhat", Vh, hb);
  // canonical code / scale / zero views, for the bit-exact comparison with the oracle
  const int ge = g ? g : 128;   // g = 0: per-vector groups, one Key group per segment, one Value pair per (head, token)
  const int ng_tot = g ? (n + g - 1) / g + nchunks * ((chunk_n + g - 1) / g) : 1 + nchunks;
  for (int which = 0; which < 2; ++which) {
    const size_t cb = (size_t)B * H * ntot * 128, sb = which == 0 ? (size_t)B * H * ng_tot * 128 * 2 : (size_t)B * H * ntot * (128 / ge) * 2;
    void *codes = aligned_alloc(256, (cb + 255) / 256 * 256), *sc = aligned_alloc(256, (sb + 255) / 256 * 256), *ze = aligned_alloc(256, (sb + 255) / 256 * 256);
    CK(gear_export_codes(&cache, which, codes, sc, ze, nullptr));
    wr(dir, which ? "Vcodes" : "Kcodes", codes, cb);
    wr(dir, which ? "Vscale" : "Kscale", sc, sb);
    wr(dir, which ? "Vzero" : "Kzero", ze, sb);
  }
  // the sparse matrix S: dense mask + values, and the coordinate form
  for (int which = 0; which < 2; ++which) {
    const size_t eb = (size_t)B * H * ntot * 128;
    void *mask = aligned_alloc(256, (eb + 255) / 256 * 256), *vals = aligned_alloc(256, (2 * eb + 255) / 256 * 256);
    CK(gear_export_sparse(&cache, which, mask, vals, nullptr));
    wr(dir, which ? "Vmask" : "Kmask", mask, eb);
    wr(dir, which ? "Vsvals" : "Ksvals", vals, 2 * eb);
    int64_t nnz = 0;
    CK(gear_export_sparse_coo(&cache, which, &nnz, nullptr, nullptr, nullptr, 0, nullptr));   // the count alone
    void *lin = aligned_alloc(256, ((size_t)nnz * 8 + 255) / 256 * 256 + 256), *cv = aligned_alloc(256, ((size_t)nnz * 2 + 255) / 256 * 256 + 256);
    CK(gear_export_sparse_coo(&cache, which, &nnz, lin, cv, work, wb, nullptr));
    wr(dir, which ? "Vcoo_idx" : "Kcoo_idx", lin, (size_t)nnz * 8);
    wr(dir, which ? "Vcoo_val" : "Kcoo_val", cv, (size_t)nnz * 2);
  }
  // the prefill segment's low-rank factors
  if (rank > 0) {
    for (int which = 0; which < 2; ++which) {
      const size_t abytes = (size_t)B * H * n * rank * 2, bbytes = (size_t)B * H * 128 * rank * 2;
      void *A = aligned_alloc(256, (abytes + 255) / 256 * 256), *Bf = aligned_alloc(256, (bbytes + 255) / 256 * 256);
      CK(gear_export_lowrank(&cache, which, 0, A, Bf, nullptr));
      wr(dir, which ? "V_A" : "K_A", A, abytes);
      wr(dir, which ? "V_B" : "K_B", Bf, bbytes);
    }
  }
  // two query rows per head over the same cache (where the kernel has the columns for them), causal
  if (2 * (Hq / H) <= 8 && n_buf >= 2) {
    void* q2 = rd(dir, "q2", -1);
    void* out2 = aligned_alloc(256, (2 * ob + 255) / 256 * 256);
    fprintf(stderr, "decode two query rows\n");
    CK(gear_decode_attn_mq(&cache, q2, 2, 1, Kb, Vb, n_buf, out2, work, wb, nullptr));
    wr(dir, "out2", out2, 2 * ob);
  }
  fprintf(stderr, "done\n");
  return 0;
}
