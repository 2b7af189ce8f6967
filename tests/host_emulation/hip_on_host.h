// Enough of the HIP device vocabulary to run a kernel on the host: one OS thread per GPU thread of a
// block with a real barrier behind __syncthreads, blocks in sequence, dynamic LDS as a heap block of
// exactly the launched size (so a sanitizer build sees any overrun).  Test infrastructure only.
#pragma once
#include <stdint.h>
#include <math.h>
#include <string.h>
#include <stdio.h>
#include <stdlib.h>
#include <algorithm>
#include <thread>
#include <vector>
#include <barrier>
#include <mutex>
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __restrict__
#define __launch_bounds__(x)
#define __shared__ static   /* one copy for the block that is running (blocks run in sequence) */
struct dim3_ { unsigned x, y, z; };
static thread_local dim3_ threadIdx, blockIdx, gridDim, blockDim;
static std::barrier<> *g_bar;
static float *g_lds;            // dynamic shared memory of the running block
#define AQT_EXTERN_LDS(name) float *name = g_lds
inline void __syncthreads() { g_bar->arrive_and_wait(); }
// wave shuffle: exchange through a per-block table
static int g_shfl[256];
inline int __shfl_xor(int v, int off, int) {
  g_shfl[threadIdx.x] = v; g_bar->arrive_and_wait();
  int r = g_shfl[threadIdx.x ^ off]; g_bar->arrive_and_wait();
  return r;
}
inline float __shfl_xor(float v, int off, int w) {
  int i; memcpy(&i, &v, 4); i = __shfl_xor(i, off, w); memcpy(&v, &i, 4); return v;
}
inline uint32_t __float_as_uint(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
inline float __uint_as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static std::mutex g_mu;
inline uint32_t atomicMax(uint32_t *p, uint32_t v) { std::lock_guard<std::mutex> l(g_mu); uint32_t o = *p; if (v > o) *p = v; return o; }
using std::max; using std::min;
inline float __builtin_amdgcn_rcpf(float d) { return 1.0f / d; }
namespace aqt {
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
}
template <class F> void run(unsigned grid, unsigned block, size_t lds_bytes, F f) {
  for (unsigned b = 0; b < grid; ++b) {
    std::barrier<> bar(block);
    g_bar = &bar;
    g_lds = (float *)malloc(lds_bytes ? lds_bytes : 4);   // exact size: ASan sees any overrun
    std::vector<std::thread> th;
    for (unsigned t = 0; t < block; ++t)
      th.emplace_back([=] { gridDim = {grid, 1, 1}; blockDim = {block, 1, 1}; blockIdx = {b, 0, 0}; threadIdx = {t, 0, 0}; f(); });
    for (auto &x : th) x.join();
    free(g_lds);
  }
}
