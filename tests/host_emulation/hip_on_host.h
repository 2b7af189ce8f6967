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
#include <memory>
#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __restrict__
#define __launch_bounds__(...)
#define __shared__ static   /* one copy for the block that is running (blocks run in sequence) */
struct dim3_ { unsigned x, y, z; };
static thread_local dim3_ threadIdx, blockIdx, gridDim, blockDim;
static std::barrier<> *g_bar;
static std::barrier<> *g_wbar[16];   // one per wavefront of the running block
static float *g_lds;            // dynamic shared memory of the running block
#define AQT_EXTERN_LDS(name) float *name = g_lds
inline void __syncthreads() { g_bar->arrive_and_wait(); }
inline void __builtin_amdgcn_wave_barrier() { g_wbar[threadIdx.x >> 6]->arrive_and_wait(); }
// wave shuffle: exchange through a table, in step with the other lanes of the wavefront
static int g_shfl[1024];
inline int __shfl_xor(int v, int off, int) {
  std::barrier<> *wb = g_wbar[threadIdx.x >> 6];
  g_shfl[threadIdx.x] = v; wb->arrive_and_wait();
  int r = g_shfl[(threadIdx.x & ~63u) | ((threadIdx.x ^ (unsigned)off) & 63u)]; wb->arrive_and_wait();
  return r;
}
// v_mfma_f32_32x32x2_f32: D = A (32 x 2) * B (2 x 32) + C; lane (lr = lane % 32, lk = lane / 32) supplies
// A[lr][lk] and B[lk][lr]; element r of its accumulator is row 8 (r / 4) + 4 lk + r % 4, column lr
struct v16f { float v[16]; float &operator[](int i) { return v[i]; } const float &operator[](int i) const { return v[i]; } };
static float g_mfa[1024], g_mfb[1024];
inline v16f __builtin_amdgcn_mfma_f32_32x32x2f32(float a, float b, v16f c, int, int, int) {
  std::barrier<> *wb = g_wbar[threadIdx.x >> 6];
  const unsigned base = threadIdx.x & ~63u, lane = threadIdx.x & 63u, lr = lane & 31u, lk = lane >> 5;
  g_mfa[threadIdx.x] = a; g_mfb[threadIdx.x] = b; wb->arrive_and_wait();
  for (int r = 0; r < 16; ++r) {
    const unsigned row = 8 * (r >> 2) + 4 * lk + (r & 3);
    c[r] = fmaf(g_mfa[base + 32 + row], g_mfb[base + 32 + lr], fmaf(g_mfa[base + row], g_mfb[base + lr], c[r]));
  }
  wb->arrive_and_wait();
  return c;
}
inline float __builtin_amdgcn_exp2f(float x) { return exp2f(x); }
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
    std::vector<std::unique_ptr<std::barrier<>>> wbars;
    for (unsigned w = 0; w * 64 < block; ++w) {
      wbars.emplace_back(new std::barrier<>(std::min(64u, block - w * 64)));
      g_wbar[w] = wbars.back().get();
    }
    g_lds = (float *)malloc(lds_bytes ? lds_bytes : 4);   // exact size: ASan sees any overrun
    std::vector<std::thread> th;
    for (unsigned t = 0; t < block; ++t)
      th.emplace_back([=] { gridDim = {grid, 1, 1}; blockDim = {block, 1, 1}; blockIdx = {b, 0, 0}; threadIdx = {t, 0, 0}; f(); });
    for (auto &x : th) x.join();
    free(g_lds);
  }
}
