// Runs the library's C ABI end to end on the CPU emulation: prefill compress, chunk compresses,
// decode attention, decompress.  Inputs and outputs are raw files in the directory given as argv[1]
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
  int B, H, Hq, bits, g, ppm, n, rank, nchunks, chunk_n, rank_chunk, n_buf, n_buf_cap, iters, flags = 0;
  char p[512]; snprintf(p, sizeof p, "%s/meta.txt", dir);
  FILE* f = fopen(p, "r");
  if (fscanf(f, "%d %d %d %d %d %d %d %d %d %d %d %d %d %d %d", &B, &H, &Hq, &bits, &g, &ppm, &n, &rank, &nchunks, &chunk_n, &rank_chunk, &n_buf, &n_buf_cap, &iters, &flags) < 14) return 1;
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
  fprintf(stderr, "done\n");
  return 0;
}
