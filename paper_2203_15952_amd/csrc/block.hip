// Pieces around the quantized dense layer that a Conformer block needs (arxiv 2203.15952,
// Sec. 3.2: feed-forward module = normalisation, Linear, Swish, Linear; Sec. 4.2 / Table 2:
// which layers run at which precision):
//   * layer normalisation fused with the per-tensor abs-max quantizer of Fig. 2, so the
//     normalised tensor is never written in float32,
//   * the chain-rule factor of the activation applied to an upstream gradient,
//   * the float32-emulated ("fake", Sec. 1) product of the integer codes on the float32
//     matrix cores, as a comparator for the native integer product,
//   * per-layer precision policies and the feed-forward module as one call.
#include "aqt_internal.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_max_u(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), off, 64));
    v = v > o ? v : o;
  }
  return v;
}

// One normalised value; both passes evaluate exactly this expression (no contraction), so
// the codes of pass 2 are codes of the very values whose maximum pass 1 took.
__device__ __forceinline__ float ln_value(float x, float mean, float rstd, const float *gamma, const float *beta,
                                          int64_t c) {
  float t = (x - mean) * rstd;
  if (gamma) t = t * gamma[c];
  if (beta) t = t + beta[c];
  return t;
}

// A row in registers: lane l keeps the float4 pieces l, l + 64, ... of its row (NV pieces, rows of up to
// 256 NV floats whose length is a multiple of 4), so each pass reads the row from memory once.
template <int NV>
__device__ __forceinline__ void load_row(const float *__restrict__ row, int64_t D, int lane, v4f (&v)[NV]) {
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int64_t c = 4 * (lane + 64 * k);
    v[k] = c < D ? *reinterpret_cast<const v4f *>(row + c) : v4f{0.0f, 0.0f, 0.0f, 0.0f};
  }
}

// Pass 1: one wavefront per row.  Row mean and biased variance in float32 (lane partial
// sums, then a fixed shuffle tree: the same bits on every run), rstd = 1 / sqrt(var + eps),
// and the largest |normalised value| of everything this block handled.
// NV > 0: the row is held in registers (D % 4 == 0, D <= 256 NV, 16-byte aligned rows); NV = 0: any row.
// When `res` is given the input row is x + alpha * res (the residual connection in front of the module:
// product, then sum, one rounding each), which is also written to `sum_out` for the second pass and the caller.
template <int NV>
__global__ __launch_bounds__(kThreads) void ln_stats_kernel(const float *__restrict__ x, int64_t M, int64_t D,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, float eps,
                                                            float *__restrict__ stats, uint32_t *__restrict__ partial,
                                                            const float *__restrict__ res, float alpha,
                                                            float *__restrict__ sum_out,
                                                            uint32_t *__restrict__ zero_word) {
  __shared__ uint32_t sm[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0u;   // for a kernel launched after this one
  uint32_t amax = 0u;
  for (int64_t m = static_cast<int64_t>(blockIdx.x) * 4 + wave; m < M; m += static_cast<int64_t>(gridDim.x) * 4) {
    const float *row = x + m * D;
    if constexpr (NV > 0) {
      v4f v[NV];
      load_row<NV>(row, D, lane, v);
      if (res) {
        v4f rv[NV];
        load_row<NV>(res + m * D, D, lane, rv);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          v[k].x = v[k].x + alpha * rv[k].x; v[k].y = v[k].y + alpha * rv[k].y;
          v[k].z = v[k].z + alpha * rv[k].z; v[k].w = v[k].w + alpha * rv[k].w;
          const int64_t c = 4 * (lane + 64 * k);
          if (c < D) *reinterpret_cast<v4f *>(sum_out + m * D + c) = v[k];
        }
      }
      float s = 0.0f;
#pragma unroll
      for (int k = 0; k < NV; ++k) s += (v[k].x + v[k].y) + (v[k].z + v[k].w);   // pieces beyond the row are zero
      const float mean = wave_sum(s) / static_cast<float>(D);
      float q = 0.0f;
#pragma unroll
      for (int k = 0; k < NV; ++k)
        if (4 * (lane + 64 * k) < D) {
          const float a = v[k].x - mean, b = v[k].y - mean, c = v[k].z - mean, d = v[k].w - mean;
          q += (a * a + b * b) + (c * c + d * d);
        }
      const float var = wave_sum(q) / static_cast<float>(D);
      const float rstd = 1.0f / sqrtf(var + eps);
      if (lane == 0) {
        stats[2 * m] = mean;
        stats[2 * m + 1] = rstd;
      }
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const int64_t c = 4 * (lane + 64 * k);
        if (c < D) {
          amax = max(amax, __float_as_uint(ln_value(v[k].x, mean, rstd, gamma, beta, c)) & 0x7FFFFFFFu);
          amax = max(amax, __float_as_uint(ln_value(v[k].y, mean, rstd, gamma, beta, c + 1)) & 0x7FFFFFFFu);
          amax = max(amax, __float_as_uint(ln_value(v[k].z, mean, rstd, gamma, beta, c + 2)) & 0x7FFFFFFFu);
          amax = max(amax, __float_as_uint(ln_value(v[k].w, mean, rstd, gamma, beta, c + 3)) & 0x7FFFFFFFu);
        }
      }
    } else {
      if (res) {   // any row length: form the sum first, then read it back like any input row
        for (int64_t c = lane; c < D; c += 64) sum_out[m * D + c] = row[c] + alpha * res[m * D + c];
        row = sum_out + m * D;
      }
      float s = 0.0f;
      for (int64_t c = lane; c < D; c += 64) s += row[c];
      const float mean = wave_sum(s) / static_cast<float>(D);
      float v = 0.0f;
      for (int64_t c = lane; c < D; c += 64) {
        const float d = row[c] - mean;
        v += d * d;
      }
      const float var = wave_sum(v) / static_cast<float>(D);
      const float rstd = 1.0f / sqrtf(var + eps);
      if (lane == 0) {
        stats[2 * m] = mean;
        stats[2 * m + 1] = rstd;
      }
      for (int64_t c = lane; c < D; c += 64)
        amax = max(amax, __float_as_uint(ln_value(row[c], mean, rstd, gamma, beta, c)) & 0x7FFFFFFFu);
    }
  }
  amax = wave_max_u(amax);
  if (lane == 0) sm[wave] = amax;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
}

__device__ __forceinline__ int8_t ln_code(float v, float s, float fq) {
  const float t = (s == 0.0f) ? 0.0f : v / s;
  float r = floorf(t + 0.5f);
  r = fminf(fmaxf(r, -fq), fq);
  return static_cast<int8_t>(static_cast<int>(r));
}

// Pass 2: fold the block maxima into the scale (Fig. 2: max / qmax), recompute the normalised
// values from x and the stored row statistics, quantize (divide, + 0.5, floor), write codes
// and, when asked, the float32 values themselves.  VEC: four columns per lane and access
// (D % 4 == 0, 16-byte aligned x and y_out, 4-byte aligned q).
template <bool VEC>
__global__ __launch_bounds__(kThreads) void ln_quantize_kernel(const float *__restrict__ x, int64_t M, int64_t D,
                                                               const float *__restrict__ gamma,
                                                               const float *__restrict__ beta,
                                                               const float *__restrict__ stats,
                                                               const uint32_t *__restrict__ partial, int nparts,
                                                               int qmax, int8_t *__restrict__ q,
                                                               float *__restrict__ scale, float *__restrict__ y_out,
                                                               int32_t *dev_status) {
  __shared__ uint32_t sm[4];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  uint32_t mx = 0u;
  for (int i = threadIdx.x; i < nparts; i += kThreads) mx = max(mx, partial[i]);
  mx = wave_max_u(mx);
  if (lane == 0) sm[wave] = mx;
  __syncthreads();
  mx = max(max(sm[0], sm[1]), max(sm[2], sm[3]));
  const float fq = static_cast<float>(qmax);
  const float s = __uint_as_float(mx) / fq;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (scale) scale[0] = s;
    if (mx >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
  for (int64_t m = static_cast<int64_t>(blockIdx.x) * 4 + wave; m < M; m += static_cast<int64_t>(gridDim.x) * 4) {
    const float *row = x + m * D;
    const float mean = stats[2 * m], rstd = stats[2 * m + 1];
    if constexpr (VEC) {
      for (int64_t c = 4 * lane; c < D; c += 256) {
        const v4f xv = *reinterpret_cast<const v4f *>(row + c);
        v4f y;
        y.x = ln_value(xv.x, mean, rstd, gamma, beta, c);
        y.y = ln_value(xv.y, mean, rstd, gamma, beta, c + 1);
        y.z = ln_value(xv.z, mean, rstd, gamma, beta, c + 2);
        y.w = ln_value(xv.w, mean, rstd, gamma, beta, c + 3);
        if (y_out) *reinterpret_cast<v4f *>(y_out + m * D + c) = y;
        if (q) {
          const uint32_t b0 = static_cast<uint8_t>(ln_code(y.x, s, fq)), b1 = static_cast<uint8_t>(ln_code(y.y, s, fq));
          const uint32_t b2 = static_cast<uint8_t>(ln_code(y.z, s, fq)), b3 = static_cast<uint8_t>(ln_code(y.w, s, fq));
          *reinterpret_cast<uint32_t *>(q + m * D + c) = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
        }
      }
    } else {
      for (int64_t c = lane; c < D; c += 64) {
        const float v = ln_value(row[c], mean, rstd, gamma, beta, c);
        if (y_out) y_out[m * D + c] = v;
        if (q) q[m * D + c] = ln_code(v, s, fq);
      }
    }
  }
}

// Backward of the normalisation.  With xh = (x - mean) rstd (statistics as the forward stored them) and
// g = dy gamma:  dx = (g - mean_row(g) - xh mean_row(g xh)) rstd (+ add, the gradient arriving over the
// residual connection), dgamma = sum_m dy xh, dbeta = sum_m dy.  One wavefront per row; each lane keeps
// column sums for its own columns over the rows its workgroup walks, the four wavefronts are added in LDS
// in a fixed order and the workgroup leaves one partial per column; ln_bwd_fold_kernel adds the partials
// in order.  NV as in ln_stats_kernel (NV = 0: any row, one column per lane and step).
template <int NV>
__global__ __launch_bounds__(kThreads) void ln_bwd_kernel(const float *__restrict__ x, const float *__restrict__ stats,
                                                          const float *__restrict__ gamma,
                                                          const float *__restrict__ dy, const float *__restrict__ add,
                                                          int64_t M, int64_t D, float *__restrict__ dx,
                                                          float *__restrict__ part) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const float invD = 1.0f / static_cast<float>(D);
  if constexpr (NV > 0) {
    __shared__ v4f sm[4][2][NV][64];
    v4f ag[NV], ab[NV], gm[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      ag[k] = ab[k] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
      const int64_t c = 4 * (lane + 64 * k);
      gm[k] = (gamma && c < D) ? *reinterpret_cast<const v4f *>(gamma + c) : v4f{1.0f, 1.0f, 1.0f, 1.0f};
    }
    for (int64_t m = static_cast<int64_t>(blockIdx.x) * 4 + wave; m < M; m += static_cast<int64_t>(gridDim.x) * 4) {
      v4f xv[NV], gv[NV];
      load_row<NV>(x + m * D, D, lane, xv);
      load_row<NV>(dy + m * D, D, lane, gv);
      const float mean = stats[2 * m], rstd = stats[2 * m + 1];
      float sg = 0.0f, sgx = 0.0f;
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const bool in = 4 * (lane + 64 * k) < D;
        v4f xh;
        xh.x = (xv[k].x - mean) * rstd; xh.y = (xv[k].y - mean) * rstd;
        xh.z = (xv[k].z - mean) * rstd; xh.w = (xv[k].w - mean) * rstd;
        if (!in) xh = v4f{0.0f, 0.0f, 0.0f, 0.0f};
        ag[k].x += gv[k].x * xh.x; ag[k].y += gv[k].y * xh.y; ag[k].z += gv[k].z * xh.z; ag[k].w += gv[k].w * xh.w;
        ab[k].x += gv[k].x; ab[k].y += gv[k].y; ab[k].z += gv[k].z; ab[k].w += gv[k].w;
        gv[k].x *= gm[k].x; gv[k].y *= gm[k].y; gv[k].z *= gm[k].z; gv[k].w *= gm[k].w;      // g = dy gamma
        sg += (gv[k].x + gv[k].y) + (gv[k].z + gv[k].w);
        sgx += (gv[k].x * xh.x + gv[k].y * xh.y) + (gv[k].z * xh.z + gv[k].w * xh.w);
        xv[k] = xh;
      }
      const float mg = wave_sum(sg) * invD, mgx = wave_sum(sgx) * invD;
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const int64_t c = 4 * (lane + 64 * k);
        if (c < D) {
          v4f o;
          o.x = (gv[k].x - mg - xv[k].x * mgx) * rstd; o.y = (gv[k].y - mg - xv[k].y * mgx) * rstd;
          o.z = (gv[k].z - mg - xv[k].z * mgx) * rstd; o.w = (gv[k].w - mg - xv[k].w * mgx) * rstd;
          if (add) {
            const v4f a = *reinterpret_cast<const v4f *>(add + m * D + c);
            o.x += a.x; o.y += a.y; o.z += a.z; o.w += a.w;
          }
          *reinterpret_cast<v4f *>(dx + m * D + c) = o;
        }
      }
    }
    if (part) {
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        sm[wave][0][k][lane] = ag[k];
        sm[wave][1][k][lane] = ab[k];
      }
      __syncthreads();
      if (wave < 2) {   // wavefront 0 folds the gamma sums, wavefront 1 the beta sums
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int64_t c = 4 * (lane + 64 * k);
          if (c < D) {
            const v4f a = sm[0][wave][k][lane], b = sm[1][wave][k][lane], c2 = sm[2][wave][k][lane], d = sm[3][wave][k][lane];
            v4f o;
            o.x = ((a.x + b.x) + c2.x) + d.x; o.y = ((a.y + b.y) + c2.y) + d.y;
            o.z = ((a.z + b.z) + c2.z) + d.z; o.w = ((a.w + b.w) + c2.w) + d.w;
            *reinterpret_cast<v4f *>(part + (static_cast<int64_t>(blockIdx.x) * 2 + wave) * D + c) = o;
          }
        }
      }
    }
  } else {
    // any row length: the row statistics of g by two passes over the row, then dx; the column sums are
    // left to ln_bwd_colsum_kernel
    for (int64_t m = static_cast<int64_t>(blockIdx.x) * 4 + wave; m < M; m += static_cast<int64_t>(gridDim.x) * 4) {
      const float mean = stats[2 * m], rstd = stats[2 * m + 1];
      float sg = 0.0f, sgx = 0.0f;
      for (int64_t c = lane; c < D; c += 64) {
        const float g = dy[m * D + c] * (gamma ? gamma[c] : 1.0f), xh = (x[m * D + c] - mean) * rstd;
        sg += g;
        sgx += g * xh;
      }
      const float mg = wave_sum(sg) * invD, mgx = wave_sum(sgx) * invD;
      for (int64_t c = lane; c < D; c += 64) {
        const float g = dy[m * D + c] * (gamma ? gamma[c] : 1.0f), xh = (x[m * D + c] - mean) * rstd;
        float o = (g - mg - xh * mgx) * rstd;
        if (add) o += add[m * D + c];
        dx[m * D + c] = o;
      }
    }
  }
}

// Any row length: partial column sums of dy xh and dy over a slab of rows, one thread per column.
__global__ __launch_bounds__(kThreads) void ln_bwd_colsum_kernel(const float *__restrict__ x,
                                                                 const float *__restrict__ stats,
                                                                 const float *__restrict__ dy, int64_t M, int64_t D,
                                                                 int64_t rows_per_slab, float *__restrict__ part) {
  const int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (c >= D) return;
  const int64_t m0 = static_cast<int64_t>(blockIdx.y) * rows_per_slab;
  const int64_t m1 = m0 + rows_per_slab < M ? m0 + rows_per_slab : M;
  float ag = 0.0f, ab = 0.0f;
  for (int64_t m = m0; m < m1; ++m) {
    const float g = dy[m * D + c];
    ag += g * ((x[m * D + c] - stats[2 * m]) * stats[2 * m + 1]);
    ab += g;
  }
  part[(static_cast<int64_t>(blockIdx.y) * 2) * D + c] = ag;
  part[(static_cast<int64_t>(blockIdx.y) * 2 + 1) * D + c] = ab;
}

__global__ __launch_bounds__(kThreads) void ln_bwd_fold_kernel(const float *__restrict__ part, int P, int64_t D,
                                                               float *__restrict__ dgamma, float *__restrict__ dbeta) {
  const int64_t c = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (c >= D) return;
  // four independent running sums per output so that loads overlap; the order of the additions is fixed
  float ag[4] = {0.0f, 0.0f, 0.0f, 0.0f}, ab[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  int p = 0;
  for (; p + 4 <= P; p += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      ag[u] += part[(static_cast<int64_t>(p + u) * 2) * D + c];
      ab[u] += part[(static_cast<int64_t>(p + u) * 2 + 1) * D + c];
    }
  }
  for (; p < P; ++p) {
    ag[0] += part[(static_cast<int64_t>(p) * 2) * D + c];
    ab[0] += part[(static_cast<int64_t>(p) * 2 + 1) * D + c];
  }
  if (dgamma) dgamma[c] = (ag[0] + ag[1]) + (ag[2] + ag[3]);
  if (dbeta) dbeta[c] = (ab[0] + ab[1]) + (ab[2] + ab[3]);
}

// out = alpha * m
__global__ __launch_bounds__(kThreads) void scale_kernel(const float *m, float alpha, float *out, int64_t n) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride) out[i] = alpha * m[i];
}

// dv[m,n] = dout[m, n mod oc] * dact[m,n]  (chain rule through the activation)
__global__ __launch_bounds__(kThreads) void dact_mul_kernel(const float *__restrict__ dout,
                                                            const float *__restrict__ dact, int64_t M, int64_t N,
                                                            int64_t oc, float *__restrict__ dv) {
  const int64_t total = M * N;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t m = i / N, n = i - m * N;
    dv[i] = dout[m * oc + (n < oc ? n : n - oc)] * dact[i];
  }
}

__global__ __launch_bounds__(kThreads) void dact_mul4_kernel(const v4f *__restrict__ dout, const v4f *__restrict__ dact,
                                                             int64_t M, int64_t N4, int64_t oc4,
                                                             v4f *__restrict__ dv) {
  const int64_t total = M * N4;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t m = i / N4, n = i - m * N4;
    const v4f a = __builtin_nontemporal_load(dout + m * oc4 + (n < oc4 ? n : n - oc4));
    const v4f b = __builtin_nontemporal_load(dact + i);
    const v4f o = {a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w};
    dv[i] = o;
  }
}

// out = x + alpha * m (the residual connection around a module); no contraction: two roundings
__global__ __launch_bounds__(kThreads) void residual_add_kernel(const float *x, const float *m, float alpha, float *out,
                                                                int64_t n) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride)
    out[i] = x[i] + alpha * m[i];
}

__global__ __launch_bounds__(kThreads) void residual_add4_kernel(const v4f *x, const v4f *m, float alpha, v4f *out,
                                                                 int64_t n4) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n4; i += stride) {
    const v4f a = x[i], b = m[i];
    const v4f o = {a.x + alpha * b.x, a.y + alpha * b.y, a.z + alpha * b.z, a.w + alpha * b.w};
    out[i] = o;
  }
}

// ---- the float32-emulated product of the codes ------------------------------------------
// "Fake" quantization on hardware without integer matrix units: the codes are converted to
// float32 and multiplied and accumulated by float32 matrix instructions
// (v_mfma_f32_32x32x2_f32).  Every product is exact; the sums are exact while they fit the
// 24-bit significand and are rounded beyond.  Tile 128 x 128 per workgroup (four
// wavefronts of 64 x 64), 32 fan-in per stage staged through LDS as bytes.
typedef float v16f __attribute__((ext_vector_type(16)));
constexpr int kFK = 32;

__global__ __launch_bounds__(kThreads) void fake_matmul_f32_kernel(const int8_t *__restrict__ xq,
                                                                   const int8_t *__restrict__ wq_kn, int M, int K,
                                                                   int N, float *__restrict__ out) {
  __shared__ int8_t sA[128][kFK + 4];   // [row][k], padded
  __shared__ int8_t sB[kFK][128 + 4];   // [k][col]
  const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
  const int wm = wave >> 1, wn = wave & 1, lr = lane & 31, lk = lane >> 5;
  const int m0 = blockIdx.y * 128, n0 = blockIdx.x * 128;
  v16f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  for (int k0 = 0; k0 < K; k0 += kFK) {
    // 128 x 32 bytes of codes: thread t loads row t/2, 16 bytes
    {
      const int r = t >> 1, c = (t & 1) * 16;
      const int gm = m0 + r;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gk = k0 + c + e;
        sA[r][c + e] = (gm < M && gk < K) ? xq[static_cast<int64_t>(gm) * K + gk] : static_cast<int8_t>(0);
      }
    }
    {
      const int r = t >> 3, c = (t & 7) * 16;
      const int gk = k0 + r;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gn = n0 + c + e;
        sB[r][c + e] = (gk < K && gn < N) ? wq_kn[static_cast<int64_t>(gk) * N + gn] : static_cast<int8_t>(0);
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kFK; kk += 2) {
      float a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = static_cast<float>(sA[wm * 64 + i * 32 + lr][kk + lk]);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = static_cast<float>(sB[kk + lk][wn * 64 + j * 32 + lr]);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int n = n0 + wn * 64 + j * 32 + lr;
        if (m < M && n < N) out[static_cast<int64_t>(m) * N + n] = acc[i][j][r];
      }
}

int grid_cap(int64_t items, int per_block, int cap) {
  int64_t g = cdiv(items, per_block);
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return static_cast<int>(g);
}

}  // namespace

size_t layernorm_ws_bytes(int64_t M) {
  return align_up(kMaxPartials * sizeof(uint32_t), 256) + align_up(static_cast<size_t>(M) * 2 * sizeof(float), 256);
}

aqt_status launch_layernorm_quantize(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                                     float eps, int bits, int8_t *q, float *scale, float *y_out, float *row_stats,
                                     void *ws, hipStream_t st, int32_t *dev_status, const float *res, float alpha,
                                     float *sum_out, uint32_t *zero_word) {
  uint32_t *partial = static_cast<uint32_t *>(ws);
  float *stats = row_stats ? row_stats
                           : reinterpret_cast<float *>(static_cast<uint8_t *>(ws) +
                                                       align_up(kMaxPartials * sizeof(uint32_t), 256));
  const int g = grid_cap(M, 4, 2048);
  const bool vec = (D % 4 == 0) && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                   (!y_out || reinterpret_cast<uintptr_t>(y_out) % 16 == 0) &&
                   (!q || reinterpret_cast<uintptr_t>(q) % 4 == 0) &&
                   (!res || (reinterpret_cast<uintptr_t>(res) % 16 == 0 && reinterpret_cast<uintptr_t>(sum_out) % 16 == 0));
  if (vec && D <= 512) ln_stats_kernel<2><<<g, kThreads, 0, st>>>(x, M, D, gamma, beta, eps, stats, partial, res, alpha, sum_out, zero_word);
  else if (vec && D <= 1024) ln_stats_kernel<4><<<g, kThreads, 0, st>>>(x, M, D, gamma, beta, eps, stats, partial, res, alpha, sum_out, zero_word);
  else ln_stats_kernel<0><<<g, kThreads, 0, st>>>(x, M, D, gamma, beta, eps, stats, partial, res, alpha, sum_out, zero_word);
  AQT_HIP(hipGetLastError());
  if (res) x = sum_out;   // the second pass normalises the sum the first pass wrote
  const int qm = q ? qmax_of(bits) : 1;
  if (vec) ln_quantize_kernel<true><<<g, kThreads, 0, st>>>(x, M, D, gamma, beta, stats, partial, g, qm, q, scale, y_out, dev_status);
  else ln_quantize_kernel<false><<<g, kThreads, 0, st>>>(x, M, D, gamma, beta, stats, partial, g, qm, q, scale, y_out, dev_status);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

constexpr int kLnBwdBlocks = 512;   // workgroups (= column-sum partials) of the normalisation's backward

size_t layernorm_bwd_ws_bytes(int64_t D) {
  return align_up(static_cast<size_t>(kLnBwdBlocks) * 2 * D * sizeof(float), 256);
}

aqt_status launch_layernorm_bwd(const float *x, const float *stats, const float *gamma, const float *dy,
                                const float *add, int64_t M, int64_t D, float *dx, float *dgamma, float *dbeta,
                                void *ws, hipStream_t st) {
  const bool want_cols = dgamma || dbeta;
  float *part = want_cols ? static_cast<float *>(ws) : nullptr;
  const bool vec = (D % 4 == 0) && D <= 1024 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(dy) % 16 == 0 && reinterpret_cast<uintptr_t>(dx) % 16 == 0 &&
                   (!add || reinterpret_cast<uintptr_t>(add) % 16 == 0) &&
                   (!gamma || reinterpret_cast<uintptr_t>(gamma) % 16 == 0);
  const int g = grid_cap(M, 4, kLnBwdBlocks);
  int P = g;
  if (vec && D <= 512) ln_bwd_kernel<2><<<g, kThreads, 0, st>>>(x, stats, gamma, dy, add, M, D, dx, part);
  else if (vec) ln_bwd_kernel<4><<<g, kThreads, 0, st>>>(x, stats, gamma, dy, add, M, D, dx, part);
  else {
    ln_bwd_kernel<0><<<g, kThreads, 0, st>>>(x, stats, gamma, dy, add, M, D, dx, nullptr);
    if (want_cols) {
      AQT_HIP(hipGetLastError());
      P = static_cast<int>(cdiv(M, 256) < kLnBwdBlocks ? cdiv(M, 256) : kLnBwdBlocks);
      const int64_t rows = cdiv(M, P);
      P = static_cast<int>(cdiv(M, rows));
      dim3 grid(static_cast<unsigned>(cdiv(D, kThreads)), static_cast<unsigned>(P));
      ln_bwd_colsum_kernel<<<grid, kThreads, 0, st>>>(x, stats, dy, M, D, rows, part);
    }
  }
  AQT_HIP(hipGetLastError());
  if (want_cols) {
    ln_bwd_fold_kernel<<<static_cast<unsigned>(cdiv(D, kThreads)), kThreads, 0, st>>>(part, P, D, dgamma, dbeta);
    AQT_HIP(hipGetLastError());
  }
  return AQT_OK;
}

aqt_status launch_scale(const float *m, float alpha, float *out, int64_t n, hipStream_t st) {
  scale_kernel<<<grid_cap(n, kThreads * 4, 4096), kThreads, 0, st>>>(m, alpha, out, n);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_dact_mul(const float *dout, const float *dact, int64_t M, int64_t N, int64_t oc, float *dv,
                           hipStream_t st) {
  const bool vec = (N % 4 == 0) && (oc % 4 == 0) && reinterpret_cast<uintptr_t>(dout) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(dact) % 16 == 0 && reinterpret_cast<uintptr_t>(dv) % 16 == 0;
  if (vec) {
    dact_mul4_kernel<<<grid_cap(M * N / 4, kThreads * 4, 4096), kThreads, 0, st>>>(
        reinterpret_cast<const v4f *>(dout), reinterpret_cast<const v4f *>(dact), M, N / 4, oc / 4,
        reinterpret_cast<v4f *>(dv));
  } else {
    dact_mul_kernel<<<grid_cap(M * N, kThreads * 4, 4096), kThreads, 0, st>>>(dout, dact, M, N, oc, dv);
  }
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_residual_add(const float *x, const float *m, float alpha, float *out, int64_t n, hipStream_t st) {
  const bool vec = (n % 4 == 0) && reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(m) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(out) % 16 == 0;
  if (vec) {
    residual_add4_kernel<<<grid_cap(n / 4, kThreads * 2, 4096), kThreads, 0, st>>>(
        reinterpret_cast<const v4f *>(x), reinterpret_cast<const v4f *>(m), alpha, reinterpret_cast<v4f *>(out), n / 4);
  } else {
    residual_add_kernel<<<grid_cap(n, kThreads * 4, 4096), kThreads, 0, st>>>(x, m, alpha, out, n);
  }
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N, float *out,
                                  hipStream_t st) {
  dim3 grid(static_cast<unsigned>(cdiv(N, 128)), static_cast<unsigned>(cdiv(M, 128)));
  fake_matmul_f32_kernel<<<grid, kThreads, 0, st>>>(xq, wq_kn, static_cast<int>(M), static_cast<int>(K),
                                                    static_cast<int>(N), out);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
