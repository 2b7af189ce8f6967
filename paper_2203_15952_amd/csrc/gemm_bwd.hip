// Straight-through backward of the quantized dense layer (arxiv 2203.15952:
// Fig. 2 holds the scale constant with stop_gradient; the rounding is passed
// straight through), for gfx950:
//   dx[m,k]  = mask_x[m,k] * sum_n (dy[m,n] * s_w[n]) * wq[k,n]
//   dw[k,n]  = mask_w[k,n] * s_x * sum_m xq[m,k] * dy[m,n]
//   dbias[n] = sum_m dy[m,n]
// A NULL mask stands for "the group's scale is non-zero".
#include "aqt_internal.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ bool mask_bit(const uint32_t *__restrict__ mask, int64_t i) {
  return (mask[i >> 5] >> (i & 31)) & 1u;
}

// ---- general kernels: one thread per output, float64 accumulation ------------------
__global__ __launch_bounds__(kThreads) void bwd_dx_general_kernel(
    const float *__restrict__ dy, const int8_t *__restrict__ wq_kn, const float *__restrict__ s_w,
    const float *__restrict__ s_x, const uint32_t *__restrict__ mask_x, int64_t M, int64_t K, int64_t N,
    float *__restrict__ dx) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (idx >= M * K) return;
  const int64_t m = idx / K, k = idx - m * K;
  double s = 0.0;
  for (int64_t n = 0; n < N; ++n)
    s += static_cast<double>(dy[m * N + n] * s_w[n]) * static_cast<double>(wq_kn[k * N + n]);
  const bool pass = mask_x ? mask_bit(mask_x, idx) : (s_x[0] != 0.0f);
  dx[idx] = pass ? static_cast<float>(s) : 0.0f;
}

__global__ __launch_bounds__(kThreads) void bwd_dw_general_kernel(
    const float *__restrict__ dy, const int8_t *__restrict__ xq, const float *__restrict__ s_x,
    const float *__restrict__ s_w, const uint32_t *__restrict__ mask_w, int64_t M, int64_t K, int64_t N,
    float *__restrict__ dw) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (idx >= K * N) return;
  const int64_t k = idx / N, n = idx - k * N;
  double s = 0.0;
  for (int64_t m = 0; m < M; ++m)
    s += static_cast<double>(xq[m * K + k]) * static_cast<double>(dy[m * N + n]);
  const bool pass = mask_w ? mask_bit(mask_w, idx) : (s_w[n] != 0.0f);
  dw[idx] = pass ? static_cast<float>(static_cast<double>(s_x[0]) * s) : 0.0f;
}

// Column sums of dy in two stages: (64 columns x row slab) partials, then a fold.
constexpr int kBiasSlabs = 64;

__global__ __launch_bounds__(kThreads) void bwd_dbias_partial_kernel(const float *__restrict__ dy, int64_t M,
                                                                     int64_t N, double *__restrict__ part) {
  __shared__ double sm[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t n = static_cast<int64_t>(blockIdx.x) * 64 + tx;
  const int64_t rows_per = cdiv(M, kBiasSlabs);
  const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per;
  const int64_t r1 = min(M, r0 + rows_per);
  double s = 0.0;
  if (n < N)
    for (int64_t r = r0 + ty; r < r1; r += 4) s += static_cast<double>(dy[r * N + n]);
  sm[ty][tx] = s;
  __syncthreads();
  if (ty == 0 && n < N) part[static_cast<int64_t>(blockIdx.y) * N + n] = (sm[0][tx] + sm[1][tx]) + (sm[2][tx] + sm[3][tx]);
}

__global__ __launch_bounds__(kThreads) void bwd_dbias_fold_kernel(const double *__restrict__ part, int64_t N,
                                                                  float *__restrict__ dbias) {
  const int64_t n = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (n >= N) return;
  double s = 0.0;
  for (int j = 0; j < kBiasSlabs; ++j) s += part[static_cast<int64_t>(j) * N + n];
  dbias[n] = static_cast<float>(s);
}

}  // namespace

size_t bwd_workspace_bytes(int64_t M, int64_t K, int64_t N) {
  (void)M;
  (void)K;
  return align_up(static_cast<size_t>(kBiasSlabs) * N * sizeof(double), 256);
}

aqt_status launch_dense_bwd(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N, float *dx,
                            float *dw, float *dbias, void *ws, size_t ws_bytes, hipStream_t st) {
  (void)ws_bytes;
  if (dx) {
    bwd_dx_general_kernel<<<static_cast<int>(cdiv(M * K, kThreads)), kThreads, 0, st>>>(
        dy, sv->wq_kn, sv->s_w, sv->s_x, sv->mask_x, M, K, N, dx);
    AQT_HIP(hipGetLastError());
  }
  if (dw) {
    bwd_dw_general_kernel<<<static_cast<int>(cdiv(K * N, kThreads)), kThreads, 0, st>>>(
        dy, sv->xq, sv->s_x, sv->s_w, sv->mask_w, M, K, N, dw);
    AQT_HIP(hipGetLastError());
  }
  if (dbias) {
    double *part = static_cast<double *>(ws);
    dim3 grid(static_cast<unsigned>(cdiv(N, 64)), kBiasSlabs);
    bwd_dbias_partial_kernel<<<grid, kThreads, 0, st>>>(dy, M, N, part);
    AQT_HIP(hipGetLastError());
    bwd_dbias_fold_kernel<<<static_cast<int>(cdiv(N, kThreads)), kThreads, 0, st>>>(part, N, dbias);
    AQT_HIP(hipGetLastError());
  }
  return AQT_OK;
}

}  // namespace aqt
