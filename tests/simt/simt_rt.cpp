// Runtime of the CPU stand-in for the HIP device environment (see hip/hip_runtime.h).
#include <hip/hip_runtime.h>
#include <vector>
#if defined(__has_feature)
#if __has_feature(memory_sanitizer)
#include <sanitizer/msan_interface.h>
#define SIMT_MSAN 1
#endif
#endif
thread_local dim3 threadIdx, blockIdx;
dim3 blockDim, gridDim;
namespace simt {
Wave waves[16];
pthread_barrier_t block_bar;
unsigned char* dyn_lds = nullptr;
extern "C" unsigned char __start_simt_lds[], __stop_simt_lds[];
static unsigned poison_seed = 12345;
static void poison_lds() {   // LDS holds whatever the previous block or kernel left: model that with garbage
#ifdef SIMT_MSAN
  __msan_poison(__start_simt_lds, __stop_simt_lds - __start_simt_lds);
  return;
#endif
  for (unsigned char* p = __start_simt_lds; p < __stop_simt_lds; ++p) { poison_seed = poison_seed * 1664525u + 1013904223u; *p = (unsigned char)(poison_seed >> 24); }
}
struct Start { int tid; dim3 b; void (*fn)(void*); void* arg; dim3 grid; };
static void* tramp_grid(void* p) {
  Start* s = (Start*)p;
  threadIdx = dim3(s->tid, 0, 0);
  for (unsigned z = 0; z < s->grid.z; ++z)
    for (unsigned y = 0; y < s->grid.y; ++y)
      for (unsigned x = 0; x < s->grid.x; ++x) {
        blockIdx = dim3(x, y, z);
        if (s->tid == 0) poison_lds();
        pthread_barrier_wait(&block_bar);
        s->fn(s->arg);
        pthread_barrier_wait(&block_bar);   // the block has finished before the next one starts
      }
  return nullptr;
}
static void spawn(int nthreads, void* (*entry)(void*), std::vector<Start>& st) {
  const int nw = (nthreads + 63) / 64;
  if (nthreads % 64 || nw > 16) { fprintf(stderr, "block size %d is not a multiple of 64\n", nthreads); abort(); }
  pthread_barrier_init(&block_bar, nullptr, nthreads);
  for (int w = 0; w < nw; ++w) pthread_barrier_init(&waves[w].bar, nullptr, 64);
  std::vector<pthread_t> th(nthreads);
  pthread_attr_t at; pthread_attr_init(&at); pthread_attr_setstacksize(&at, 1 << 20);
  for (int i = 0; i < nthreads; ++i) pthread_create(&th[i], &at, entry, &st[i]);
  for (int i = 0; i < nthreads; ++i) pthread_join(th[i], nullptr);
  for (int w = 0; w < nw; ++w) pthread_barrier_destroy(&waves[w].bar);
  pthread_barrier_destroy(&block_bar);
}
void launch_grid(dim3 grid, dim3 block, size_t lds, void (*fn)(void*), void* arg) {
  if (block.y != 1 || block.z != 1) { fprintf(stderr, "only 1-D blocks are modelled\n"); abort(); }
  gridDim = grid; blockDim = block;
  // exact-size heap buffer: the address sanitizer flags any access past the requested LDS size
  dyn_lds = lds ? (unsigned char*)aligned_alloc(16, (lds + 15) / 16 * 16) : nullptr;
#ifndef SIMT_MSAN   // under the memory sanitizer fresh heap memory already counts as uninitialised
  for (size_t i = 0; i < lds; ++i) { poison_seed = poison_seed * 1664525u + 1013904223u; dyn_lds[i] = (unsigned char)(poison_seed >> 24); }
#endif
  std::vector<Start> st(block.x);
  for (unsigned i = 0; i < block.x; ++i) st[i] = Start{(int)i, dim3(), fn, arg, grid};
  spawn((int)block.x, tramp_grid, st);
  free(dyn_lds);
  dyn_lds = nullptr;
}
}  // namespace simt
