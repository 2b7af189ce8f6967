// Abs-max quantizers of native QAT (arxiv 2203.15952, Fig. 2 and Sec. 2.2) for gfx950.
//
// Per reduction group: m = max|x|, scale = m / qmax, code = floor(x / scale + 0.5)
// with x / scale replaced by 0 when scale is 0.  Every operation is a single
// float32 rounding (IEEE divide, separate add), so codes and scales are
// reproducible bit for bit.  The kernels are bound by HBM traffic: the
// per-tensor path reads the tensor twice (reduce, then quantize; the second pass
// walks the tensor backwards, so what the first pass touched last is read first)
// and writes one byte per element.
#include "aqt_internal.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// For non-negative floats the unsigned order of the bit patterns is the numeric
// order, with +Inf and NaN above every finite value: one integer max both
// reduces and detects non-finite input.
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), off, 64));
    v = v > o ? v : o;
  }
  return v;
}

// Max over a 256-thread block, result valid in every thread.
__device__ __forceinline__ uint32_t block_max(uint32_t v, uint32_t *sm /*[4]*/) {
  v = wave_max(v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[wave] = v;
  __syncthreads();
  uint32_t a = sm[0], b = sm[1], c = sm[2], d = sm[3];
  a = a > b ? a : b;
  c = c > d ? c : d;
  return a > c ? a : c;
}

// The element-wise part of Fig. 2.  fq = (float)qmax.
__device__ __forceinline__ int quant_code(float x, float s, float fq, bool &pass) {
  float t = (s == 0.0f) ? 0.0f : x / s;
  float u = t + 0.5f;
  float r = floorf(u);
  pass = (r >= -fq) && (r <= fq) && (s != 0.0f);
  r = fminf(fmaxf(r, -fq), fq);
  return static_cast<int>(r);
}

__device__ __forceinline__ int quant_code(float x, float s, float fq) {
  bool p;
  return quant_code(x, s, fq, p);
}

// Streaming 16-byte accesses.  The non-temporal hint keeps a tensor that is read
// once per pass from displacing everything else in the caches; on this part it is
// also what lets a pure stream reach its best HBM rate.
typedef float v4f __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4 *p) {
  const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(uint32_t *p, uint32_t v) { __builtin_nontemporal_store(v, p); }

__device__ __forceinline__ uint32_t absmax4(float4 a) {
  return max(max(abs_bits(a.x), abs_bits(a.y)), max(abs_bits(a.z), abs_bits(a.w)));
}

// ---- per-tensor, contiguous: pass 1 -------------------------------------------
// Each block owns one contiguous run of the tensor (per4 float4 per block).
template <bool STREAM>
__global__ __launch_bounds__(kThreads) void absmax_flat_kernel(const float *__restrict__ x, int64_t n,
                                                               int64_t per4, uint32_t *__restrict__ partial) {
  auto ld = [](const float4 *p) { return STREAM ? load_stream(p) : *p; };
  __shared__ uint32_t sm[4];
  const int64_t n4 = n >> 2;
  const float4 *x4 = reinterpret_cast<const float4 *>(x);
  const int64_t i0 = static_cast<int64_t>(blockIdx.x) * per4;
  const int64_t i1 = min(n4, i0 + per4);
  uint32_t m = 0;
  int64_t i = i0 + threadIdx.x;
  for (; i + 3 * kThreads < i1; i += 4 * kThreads) {
    const float4 a = ld(x4 + i), b = ld(x4 + i + kThreads);
    const float4 c = ld(x4 + i + 2 * kThreads), d = ld(x4 + i + 3 * kThreads);
    m = max(m, max(max(absmax4(a), absmax4(b)), max(absmax4(c), absmax4(d))));
  }
  for (; i < i1; i += kThreads) m = max(m, absmax4(ld(x4 + i)));
  if (blockIdx.x == 0)
    for (int64_t j = (n4 << 2) + threadIdx.x; j < n; j += kThreads) m = max(m, abs_bits(x[j]));
  m = block_max(m, sm);
  if (threadIdx.x == 0) partial[blockIdx.x] = m;
}

__device__ __forceinline__ uint32_t pack4(float4 v, float s, float fq) {
  uint32_t c0 = static_cast<uint32_t>(quant_code(v.x, s, fq)) & 0xFFu;
  uint32_t c1 = static_cast<uint32_t>(quant_code(v.y, s, fq)) & 0xFFu;
  uint32_t c2 = static_cast<uint32_t>(quant_code(v.z, s, fq)) & 0xFFu;
  uint32_t c3 = static_cast<uint32_t>(quant_code(v.w, s, fq)) & 0xFFu;
  return c0 | (c1 << 8) | (c2 << 16) | (c3 << 24);
}

// ---- per-tensor, contiguous: pass 2 -------------------------------------------
// Same block -> run mapping as pass 1, but blocks are visited in reverse so that
// the part of the tensor pass 1 touched last is read first.
__global__ __launch_bounds__(kThreads) void quantize_flat_kernel(
    const float *__restrict__ x, int64_t n, int64_t per4, const uint32_t *__restrict__ partial, int nparts,
    int qmax, int8_t *__restrict__ q, float *__restrict__ scale, int32_t *dev_status) {
  __shared__ uint32_t sm[4];
  uint32_t m = 0;
  for (int i = threadIdx.x; i < nparts; i += kThreads) m = max(m, partial[i]);
  m = block_max(m, sm);
  const float fq = static_cast<float>(qmax);
  const float s = __uint_as_float(m) / fq;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    scale[0] = s;
    if (m >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
  const int64_t n4 = n >> 2;
  const float4 *x4 = reinterpret_cast<const float4 *>(x);
  uint32_t *q4 = reinterpret_cast<uint32_t *>(q);
  const int64_t blk = static_cast<int64_t>(gridDim.x) - 1 - blockIdx.x;
  const int64_t i0 = blk * per4;
  const int64_t i1 = min(n4, i0 + per4);
  int64_t i = i0 + threadIdx.x;
  for (; i + 3 * kThreads < i1; i += 4 * kThreads) {
    const float4 a = load_stream(x4 + i), b = load_stream(x4 + i + kThreads);
    const float4 c = load_stream(x4 + i + 2 * kThreads), d = load_stream(x4 + i + 3 * kThreads);
    store_stream(q4 + i, pack4(a, s, fq));
    store_stream(q4 + i + kThreads, pack4(b, s, fq));
    store_stream(q4 + i + 2 * kThreads, pack4(c, s, fq));
    store_stream(q4 + i + 3 * kThreads, pack4(d, s, fq));
  }
  for (; i < i1; i += kThreads) store_stream(q4 + i, pack4(load_stream(x4 + i), s, fq));
  if (blockIdx.x == 0)
    for (int64_t j = (n4 << 2) + threadIdx.x; j < n; j += kThreads) q[j] = static_cast<int8_t>(quant_code(x[j], s, fq));
}

// ---- general shapes: abs-max per tensor / column / row ---------------------------
__global__ __launch_bounds__(kThreads) void absmax_strided_kernel(const float *__restrict__ x, int64_t rows,
                                                                  int64_t cols, int64_t ldx,
                                                                  uint32_t *__restrict__ partial) {
  __shared__ uint32_t sm[4];
  uint32_t m = 0;
  const int64_t n = rows * cols;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride) {
    const int64_t r = i / cols, c = i - r * cols;
    m = max(m, abs_bits(x[r * ldx + c]));
  }
  m = block_max(m, sm);
  if (threadIdx.x == 0) partial[blockIdx.x] = m;
}

// Reduce the per-block maxima into the single scale (and the non-finite flag).
__global__ __launch_bounds__(kThreads) void finish_scale_all_kernel(const uint32_t *__restrict__ partial,
                                                                    int nparts, int qmax,
                                                                    float *__restrict__ scale,
                                                                    int32_t *dev_status) {
  __shared__ uint32_t sm[4];
  uint32_t m = 0;
  for (int i = threadIdx.x; i < nparts; i += kThreads) m = max(m, partial[i]);
  m = block_max(m, sm);
  if (threadIdx.x == 0) {
    scale[0] = __uint_as_float(m) / static_cast<float>(qmax);
    if (m >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
}

// One scale per column: 64 columns per block, 4 row lanes.
__global__ __launch_bounds__(kThreads) void scale_cols_kernel(const float *__restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ldx, int qmax,
                                                              float *__restrict__ scale,
                                                              int32_t *dev_status) {
  __shared__ uint32_t sm[4][64];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t c = static_cast<int64_t>(blockIdx.x) * 64 + tx;
  uint32_t m = 0;
  if (c < cols)
    for (int64_t r = ty; r < rows; r += 4) m = max(m, abs_bits(x[r * ldx + c]));
  sm[ty][tx] = m;
  __syncthreads();
  if (ty == 0 && c < cols) {
    m = max(max(sm[0][tx], sm[1][tx]), max(sm[2][tx], sm[3][tx]));
    scale[c] = __uint_as_float(m) / static_cast<float>(qmax);
    if (m >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
}

// One scale per row: one wavefront per row.
__global__ __launch_bounds__(kThreads) void scale_rows_kernel(const float *__restrict__ x, int64_t rows,
                                                              int64_t cols, int64_t ldx, int qmax,
                                                              float *__restrict__ scale,
                                                              int32_t *dev_status) {
  const int lane = threadIdx.x & 63;
  const int64_t r = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  uint32_t m = 0;
  for (int64_t c = lane; c < cols; c += 64) m = max(m, abs_bits(x[r * ldx + c]));
  m = wave_max(m);
  if (lane == 0) {
    scale[r] = __uint_as_float(m) / static_cast<float>(qmax);
    if (m >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
}

// Element-wise half for any axis / stride / mask: one thread per 32 consecutive
// elements (one mask word).
__global__ __launch_bounds__(kThreads) void quantize_elem_kernel(const float *__restrict__ x, int64_t rows,
                                                                 int64_t cols, int64_t ldx, int qmax,
                                                                 int axis, const float *__restrict__ scale,
                                                                 int8_t *__restrict__ q,
                                                                 uint32_t *__restrict__ mask) {
  const int64_t n = rows * cols;
  const int64_t w = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t i0 = w * 32;
  if (i0 >= n) return;
  const float fq = static_cast<float>(qmax);
  int64_t r = i0 / cols, c = i0 - r * cols;
  uint32_t bits = 0;
  const int cnt = static_cast<int>(min(static_cast<int64_t>(32), n - i0));
  for (int j = 0; j < cnt; ++j) {
    const float s = (axis == AQT_AXIS_ALL) ? scale[0] : (axis == AQT_AXIS_ROWS ? scale[c] : scale[r]);
    bool pass;
    q[i0 + j] = static_cast<int8_t>(quant_code(x[r * ldx + c], s, fq, pass));
    bits |= static_cast<uint32_t>(pass) << j;
    if (++c == cols) { c = 0; ++r; }
  }
  if (mask) mask[w] = bits;
}

// ---- weights: per output channel, emit the forward operand ------------------------
// Two launches.  (1) abs-max of every column over a slab of fan-in rows: 64
// columns x 4 row lanes per block, grid (column blocks, slabs).  (2) one block per
// 32-channel x 64-fan-in tile folds the slab maxima of its channels into the scale,
// quantizes the tile, writes the [K,N] codes, transposes the tile through LDS and
// writes fan-in-contiguous rows, packed two codes per byte when bits_w <= 4.
constexpr int kWCols = 32;
constexpr int kWChunk = 64;

__device__ __forceinline__ void wabsmax_partial_body(const float *__restrict__ w, int64_t K, int64_t N,
                                                     int64_t rows_per_slab, int vec4, uint32_t *__restrict__ part,
                                                     unsigned bx, unsigned by) {
  __shared__ uint32_t sm[16][64];
  const int64_t k0 = static_cast<int64_t>(by) * rows_per_slab;
  const int64_t k1 = min(K, k0 + rows_per_slab);
  if (vec4) {
    // 16 column groups of 4 x 16 row lanes; four independent 16-byte loads in flight per
    // thread (the matrix is small, so the pass is bound by load latency, not bandwidth)
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t n = static_cast<int64_t>(bx) * 64 + tx * 4;
    uint32_t m0 = 0, m1 = 0, m2 = 0, m3 = 0;
    if (n < N) {
      const float4 zero = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
      for (int64_t k = k0 + ty; k < k1; k += 64) {
        const float4 a = *reinterpret_cast<const float4 *>(w + k * N + n);
        const float4 b = (k + 16 < k1) ? *reinterpret_cast<const float4 *>(w + (k + 16) * N + n) : zero;
        const float4 c = (k + 32 < k1) ? *reinterpret_cast<const float4 *>(w + (k + 32) * N + n) : zero;
        const float4 d = (k + 48 < k1) ? *reinterpret_cast<const float4 *>(w + (k + 48) * N + n) : zero;
        m0 = max(max(m0, abs_bits(a.x)), max(max(abs_bits(b.x), abs_bits(c.x)), abs_bits(d.x)));
        m1 = max(max(m1, abs_bits(a.y)), max(max(abs_bits(b.y), abs_bits(c.y)), abs_bits(d.y)));
        m2 = max(max(m2, abs_bits(a.z)), max(max(abs_bits(b.z), abs_bits(c.z)), abs_bits(d.z)));
        m3 = max(max(m3, abs_bits(a.w)), max(max(abs_bits(b.w), abs_bits(c.w)), abs_bits(d.w)));
      }
    }
    sm[ty][tx * 4 + 0] = m0; sm[ty][tx * 4 + 1] = m1; sm[ty][tx * 4 + 2] = m2; sm[ty][tx * 4 + 3] = m3;
    __syncthreads();
    if (threadIdx.x < 64) {
      const int64_t nn = static_cast<int64_t>(bx) * 64 + threadIdx.x;
      uint32_t m = 0;
#pragma unroll
      for (int j = 0; j < 16; ++j) m = max(m, sm[j][threadIdx.x]);
      if (nn < N) part[static_cast<int64_t>(by) * N + nn] = m;
    }
    return;
  }
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int64_t n = static_cast<int64_t>(bx) * 64 + tx;
  uint32_t m = 0;
  if (n < N)
    for (int64_t k = k0 + ty; k < k1; k += 4) m = max(m, abs_bits(w[k * N + n]));
  sm[ty][tx] = m;
  __syncthreads();
  if (ty == 0 && n < N)
    part[static_cast<int64_t>(by) * N + n] = max(max(sm[0][tx], sm[1][tx]), max(sm[2][tx], sm[3][tx]));
}

__global__ __launch_bounds__(kThreads) void wabsmax_partial_kernel(const float *__restrict__ w, int64_t K,
                                                                   int64_t N, int64_t rows_per_slab, int vec4,
                                                                   uint32_t *__restrict__ part) {
  wabsmax_partial_body(w, K, N, rows_per_slab, vec4, part, blockIdx.x, blockIdx.y);
}

__device__ __forceinline__ void quantize_weights_body(
    const float *__restrict__ w, int64_t K, int64_t N, int qmax, int packed, const uint32_t *__restrict__ part,
    int slabs, uint8_t *__restrict__ wq_packed, float *__restrict__ s_w, int8_t *__restrict__ wq_kn,
    uint32_t *__restrict__ mask_w, int32_t *dev_status, uint4 *__restrict__ wfrag, unsigned bx, unsigned by) {
  __shared__ int8_t tile[kWCols][kWChunk + 4];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int64_t n0 = static_cast<int64_t>(bx) * kWCols;
  const int64_t k0 = static_cast<int64_t>(by) * kWChunk;
  const int64_t n = n0 + tx;
  const bool live = n < N;
  uint32_t m = 0;
  if (live)
    for (int j = 0; j < slabs; ++j) m = max(m, part[static_cast<int64_t>(j) * N + n]);
  const float fq = static_cast<float>(qmax);
  const float s = __uint_as_float(m) / fq;
  if (by == 0 && ty == 0 && live) {
    s_w[n] = s;
    if (m >= 0x7F800000u && dev_status) *dev_status = AQT_ERR_NONFINITE;
  }
  const int64_t row_bytes = packed ? (K + 1) / 2 : K;
#pragma unroll
  for (int j = 0; j < kWChunk / 8; ++j) {
    const int kk = ty + 8 * j;
    const int64_t k = k0 + kk;
    int code = 0;
    if (live && k < K) {
      bool pass;
      code = quant_code(w[k * N + n], s, fq, pass);
      if (wq_kn) wq_kn[k * N + n] = static_cast<int8_t>(code);
      // Mask words straddle threads here; bits are set with an atomic OR on a
      // buffer the launcher has zeroed.
      if (mask_w && pass) atomicOr(&mask_w[(k * N + n) >> 5], 1u << ((k * N + n) & 31));
    }
    tile[tx][kk] = static_cast<int8_t>(code);
  }
  __syncthreads();
  // 32 rows x (64 | 32) output bytes; thread t handles bytes t, t+256, ...
  const int bytes_per_row = packed ? kWChunk / 2 : kWChunk;
  for (int b = threadIdx.x; b < kWCols * bytes_per_row; b += kThreads) {
    const int rn = b / bytes_per_row, jb = b - rn * bytes_per_row;
    const int64_t nn = n0 + rn;
    if (nn >= N) continue;
    if (packed) {
      const int64_t kb = (k0 >> 1) + jb;
      if (kb < row_bytes) {
        const uint32_t lo = static_cast<uint32_t>(tile[rn][2 * jb]) & 0xFu;
        const uint32_t hi = static_cast<uint32_t>(tile[rn][2 * jb + 1]) & 0xFu;  // 0 beyond K
        wq_packed[nn * row_bytes + kb] = static_cast<uint8_t>(lo | (hi << 4));
      }
    } else {
      const int64_t k = k0 + jb;
      if (k < K) wq_packed[nn * row_bytes + k] = static_cast<uint8_t>(tile[rn][jb]);
    }
  }
  // The same tile once more in the order the forward contraction's matrix-core fragments
  // want it (see weights_to_frag_kernel in gemm_fwd.hip for the layout), so that the
  // forward needs no re-ordering pass of its own.  Only requested for whole tiles
  // (N % 32 == 0, K % 64 == 0).  This block's tile is exactly one packed fragment (32
  // channels x two 32-deep steps) or two int8 fragments.
  if (wfrag) {
    const int lane = threadIdx.x & 63, lr = lane & 31, lk = lane >> 5;
    if (packed) {
      if (threadIdx.x < 64) {
        uint32_t d[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {          // dword q: step q / 2, codes 8 * (q % 2) .. + 7 of this lane's 16
          const int kb = 32 * (q >> 1) + 16 * lk + 8 * (q & 1);
          uint32_t t = 0;
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const uint32_t lo = static_cast<uint32_t>(tile[lr][kb + b]) & 0xFu;
            const uint32_t hi = static_cast<uint32_t>(tile[lr][kb + 4 + b]) & 0xFu;
            t |= (lo | (hi << 4)) << (8 * b);
          }
          d[q] = t;
        }
        const int64_t frag = static_cast<int64_t>(bx) * (K / 64) + by;
        wfrag[frag * 64 + lane] = make_uint4(d[0], d[1], d[2], d[3]);
      }
    } else if (threadIdx.x < 128) {
      const int h = threadIdx.x >> 6;           // which of the tile's two steps
      uint32_t d[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t t = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b)
          t |= (static_cast<uint32_t>(tile[lr][32 * h + 16 * lk + 4 * q + b]) & 0xFFu) << (8 * b);
        d[q] = t;
      }
      const int64_t frag = static_cast<int64_t>(bx) * (K / 32) + 2 * by + h;
      wfrag[frag * 64 + lane] = make_uint4(d[0], d[1], d[2], d[3]);
    }
  }
}

__global__ __launch_bounds__(kThreads) void quantize_weights_kernel(
    const float *__restrict__ w, int64_t K, int64_t N, int qmax, int packed, const uint32_t *__restrict__ part,
    int slabs, uint8_t *__restrict__ wq_packed, float *__restrict__ s_w, int8_t *__restrict__ wq_kn,
    uint32_t *__restrict__ mask_w, int32_t *dev_status, uint4 *__restrict__ wfrag) {
  quantize_weights_body(w, K, N, qmax, packed, part, slabs, wq_packed, s_w, wq_kn, mask_w, dev_status, wfrag,
                        blockIdx.x, blockIdx.y);
}

// Several weight matrices in one launch pair: a one-dimensional grid holds every matrix's own blocks one matrix
// after the other (first1 / first2: where each matrix's blocks start).  The arithmetic per matrix is that of the
// single-matrix kernels above.
struct WeightJobDev {
  const float *w;
  int64_t K, N, rows_per_slab;
  int qmax, packed, slabs, vec4;
  unsigned gx1, gx2;          // this matrix's own grid width: abs-max column blocks, quantizer column blocks
  uint32_t *part;
  uint8_t *wq_packed;
  float *s_w;
  int8_t *wq_kn;
  uint32_t *mask_w;
  uint4 *wfrag;
};
struct WeightJobsDev {
  WeightJobDev job[kWeightJobsMax];
  unsigned first1[kWeightJobsMax + 1], first2[kWeightJobsMax + 1];   // block offsets; entries from n on: the grid size
  int n;
};

// Which matrix a block belongs to (first[] ascends, first[0] = 0, blockIdx.x < first[n]).
__device__ __forceinline__ int job_of_block(const unsigned *first, int n, unsigned b) {
  int j = 0;
#pragma unroll
  for (int i = 1; i < kWeightJobsMax; ++i) j += (i < n && b >= first[i]) ? 1 : 0;
  return j;
}

__global__ __launch_bounds__(kThreads) void wabsmax_partial_group_kernel(const WeightJobsDev jobs) {
  const int ji = job_of_block(jobs.first1, jobs.n, blockIdx.x);
  const WeightJobDev &j = jobs.job[ji];
  const unsigned local = blockIdx.x - jobs.first1[ji];
  wabsmax_partial_body(j.w, j.K, j.N, j.rows_per_slab, j.vec4, j.part, local % j.gx1, local / j.gx1);
}

__global__ __launch_bounds__(kThreads) void quantize_weights_group_kernel(const WeightJobsDev jobs,
                                                                          int32_t *dev_status) {
  const int ji = job_of_block(jobs.first2, jobs.n, blockIdx.x);
  const WeightJobDev &j = jobs.job[ji];
  const unsigned local = blockIdx.x - jobs.first2[ji];
  quantize_weights_body(j.w, j.K, j.N, j.qmax, j.packed, j.part, j.slabs, j.wq_packed, j.s_w, j.wq_kn, j.mask_w,
                        dev_status, j.wfrag, local % j.gx2, local / j.gx2);
}

__global__ __launch_bounds__(kThreads) void zero_words_kernel(uint32_t *p, int64_t n) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n; i += stride) p[i] = 0;
}

__global__ __launch_bounds__(kThreads) void unpack_weights_kernel(const uint8_t *__restrict__ wq_packed,
                                                                  int64_t K, int64_t N, int packed,
                                                                  int8_t *__restrict__ codes_kn) {
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i >= K * N) return;
  const int64_t k = i / N, n = i - k * N;
  int code;
  if (packed) {
    const uint32_t b = wq_packed[n * ((K + 1) / 2) + (k >> 1)];
    const uint32_t nib = (k & 1) ? (b >> 4) : (b & 0xFu);
    code = static_cast<int>(nib ^ 8u) - 8;  // sign-extend the nibble
  } else {
    code = static_cast<int8_t>(wq_packed[n * K + k]);
  }
  codes_kn[i] = static_cast<int8_t>(code);
}

int grid_for(int64_t work_items, int per_block, int cap) {
  int64_t g = cdiv(work_items, per_block);
  if (g < 1) g = 1;
  if (g > cap) g = cap;
  return static_cast<int>(g);
}

}  // namespace

aqt_status launch_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int axis,
                           int8_t *q, float *scale, uint32_t *mask, float *partials, hipStream_t st,
                           int32_t *dev_status) {
  const int qmax = qmax_of(bits);
  const int64_t n = rows * cols;
  uint32_t *part = reinterpret_cast<uint32_t *>(partials);
  if (axis == AQT_AXIS_ALL) {
    const bool flat = (ldx == cols) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                      (reinterpret_cast<uintptr_t>(q) % 4 == 0);
    if (flat && !mask) {
      // up to 4096 blocks = 16 per CU, each on its own contiguous run of the tensor;
      // every thread keeps four 16-byte loads in flight.
      int g = grid_for(n / 4, kThreads * 4, kMaxPartials);
      const int64_t per4 = cdiv(cdiv(n / 4, g), kThreads) * kThreads;
      g = static_cast<int>(per4 > 0 ? cdiv(n / 4, per4) : 1);
      if (g < 1) g = 1;
      // Below 192 MB pass 1 reads with ordinary loads, above with non-temporal ones: measured,
      // ordinary loads make the pair of passes 2-5 % faster at 26, 105 and 134 MB (whether that
      // is the second pass hitting a cache is not something the available counters can show).
      if (n * 4 <= (int64_t(192) << 20)) absmax_flat_kernel<false><<<g, kThreads, 0, st>>>(x, n, per4, part);
      else absmax_flat_kernel<true><<<g, kThreads, 0, st>>>(x, n, per4, part);
      AQT_HIP(hipGetLastError());
      quantize_flat_kernel<<<g, kThreads, 0, st>>>(x, n, per4, part, g, qmax, q, scale, dev_status);
      AQT_HIP(hipGetLastError());
      return AQT_OK;
    }
    int g = grid_for(n, kThreads * 8, 2048);
    if (flat) {
      const int64_t per4 = cdiv(cdiv(n / 4 > 0 ? n / 4 : 1, g), kThreads) * kThreads;
      g = static_cast<int>(cdiv(n / 4 > 0 ? n / 4 : 1, per4));
      absmax_flat_kernel<true><<<g, kThreads, 0, st>>>(x, n, per4, part);
    } else
      absmax_strided_kernel<<<g, kThreads, 0, st>>>(x, rows, cols, ldx, part);
    AQT_HIP(hipGetLastError());
    finish_scale_all_kernel<<<1, kThreads, 0, st>>>(part, g, qmax, scale, dev_status);
    AQT_HIP(hipGetLastError());
  } else if (axis == AQT_AXIS_ROWS) {
    scale_cols_kernel<<<static_cast<int>(cdiv(cols, 64)), kThreads, 0, st>>>(x, rows, cols, ldx, qmax, scale,
                                                                             dev_status);
    AQT_HIP(hipGetLastError());
  } else {
    scale_rows_kernel<<<static_cast<int>(cdiv(rows, 4)), kThreads, 0, st>>>(x, rows, cols, ldx, qmax, scale,
                                                                            dev_status);
    AQT_HIP(hipGetLastError());
  }
  return launch_quantize_with_scale(x, rows, cols, ldx, bits, axis, scale, q, mask, st);
}

// Per tensor with the abs-max already known (its bit pattern in device memory): the
// single word stands in for the array of per-block maxima, so this is pass 2 alone.
aqt_status launch_quantize_with_absmax(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                       const uint32_t *absmax_bits, int8_t *q, float *scale, uint32_t *mask,
                                       hipStream_t st, int32_t *dev_status) {
  const int qmax = qmax_of(bits);
  const int64_t n = rows * cols;
  const bool flat = (ldx == cols) && (reinterpret_cast<uintptr_t>(x) % 16 == 0) &&
                    (reinterpret_cast<uintptr_t>(q) % 4 == 0);
  if (flat && !mask) {
    int g = grid_for(n / 4, kThreads * 4, kMaxPartials);
    const int64_t per4 = cdiv(cdiv(n / 4, g), kThreads) * kThreads;
    g = static_cast<int>(per4 > 0 ? cdiv(n / 4, per4) : 1);
    if (g < 1) g = 1;
    quantize_flat_kernel<<<g, kThreads, 0, st>>>(x, n, per4, absmax_bits, 1, qmax, q, scale, dev_status);
    AQT_HIP(hipGetLastError());
    return AQT_OK;
  }
  finish_scale_all_kernel<<<1, kThreads, 0, st>>>(absmax_bits, 1, qmax, scale, dev_status);
  AQT_HIP(hipGetLastError());
  return launch_quantize_with_scale(x, rows, cols, ldx, bits, AQT_AXIS_ALL, scale, q, mask, st);
}

aqt_status launch_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                      int axis, const float *scale, int8_t *q, uint32_t *mask,
                                      hipStream_t st) {
  const int64_t words = cdiv(rows * cols, 32);
  quantize_elem_kernel<<<static_cast<int>(cdiv(words, kThreads)), kThreads, 0, st>>>(
      x, rows, cols, ldx, qmax_of(bits), axis, scale, q, mask);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_quantize_weights(const float *w, int64_t K, int64_t N, int bits_w, void *wq_packed,
                                   float *s_w, int8_t *wq_kn, uint32_t *mask_w, uint32_t *part, hipStream_t st,
                                   int32_t *dev_status, void *wfrag) {
  if (wfrag && (N % kWCols != 0 || K % kWChunk != 0 || reinterpret_cast<uintptr_t>(wfrag) % 16 != 0))
    return AQT_ERR_INVALID_ARG;
  if (mask_w) {
    const int64_t words = cdiv(K * N, 32);
    zero_words_kernel<<<grid_for(words, kThreads, 1024), kThreads, 0, st>>>(mask_w, words);
    AQT_HIP(hipGetLastError());
  }
  int64_t slabs = cdiv(K, 32);
  if (slabs > kWeightSlabs) slabs = kWeightSlabs;
  const int64_t rows_per_slab = cdiv(K, slabs);
  slabs = cdiv(K, rows_per_slab);
  dim3 g1(static_cast<unsigned>(cdiv(N, 64)), static_cast<unsigned>(slabs));
  const int vec4 = (N % 4 == 0) && (reinterpret_cast<uintptr_t>(w) % 16 == 0);
  wabsmax_partial_kernel<<<g1, kThreads, 0, st>>>(w, K, N, rows_per_slab, vec4, part);
  AQT_HIP(hipGetLastError());
  dim3 g2(static_cast<unsigned>(cdiv(N, kWCols)), static_cast<unsigned>(cdiv(K, kWChunk)));
  quantize_weights_kernel<<<g2, kThreads, 0, st>>>(w, K, N, qmax_of(bits_w), packed4(bits_w) ? 1 : 0, part,
                                                   static_cast<int>(slabs), static_cast<uint8_t *>(wq_packed),
                                                   s_w, wq_kn, mask_w, dev_status, static_cast<uint4 *>(wfrag));
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_quantize_weights_group(const WeightJob *jobs, int n, hipStream_t st, int32_t *dev_status) {
  if (n < 0 || n > kWeightJobsMax) return AQT_ERR_INVALID_ARG;
  if (n == 0) return AQT_OK;
  if (n == 1)
    return launch_quantize_weights(jobs[0].w, jobs[0].K, jobs[0].N, jobs[0].bits_w, jobs[0].wq_packed, jobs[0].s_w,
                                   jobs[0].wq_kn, jobs[0].mask_w, jobs[0].part, st, dev_status, jobs[0].wfrag);
  WeightJobsDev d;
  uint64_t b1 = 0, b2 = 0;     // blocks so far in the two grids
  for (int i = 0; i < n; ++i) {
    const WeightJob &a = jobs[i];
    if (!a.w || !a.wq_packed || !a.s_w || !a.part || a.K < 1 || a.N < 1) return AQT_ERR_INVALID_ARG;
    if (a.wfrag && (a.N % kWCols != 0 || a.K % kWChunk != 0 || reinterpret_cast<uintptr_t>(a.wfrag) % 16 != 0))
      return AQT_ERR_INVALID_ARG;
    if (cdiv(a.N, kWCols) * cdiv(a.K, kWChunk) > 0x0FFFFFFF) return AQT_ERR_UNSUPPORTED;   // 8 of them stay under 2^31
    if (a.mask_w) {
      const int64_t words = cdiv(a.K * a.N, 32);
      zero_words_kernel<<<grid_for(words, kThreads, 1024), kThreads, 0, st>>>(a.mask_w, words);
      AQT_HIP(hipGetLastError());
    }
    int64_t slabs = cdiv(a.K, 32);
    if (slabs > kWeightSlabs) slabs = kWeightSlabs;
    const int64_t rows_per_slab = cdiv(a.K, slabs);
    slabs = cdiv(a.K, rows_per_slab);
    WeightJobDev &j = d.job[i];
    j.w = a.w; j.K = a.K; j.N = a.N; j.rows_per_slab = rows_per_slab;
    j.qmax = qmax_of(a.bits_w); j.packed = packed4(a.bits_w) ? 1 : 0; j.slabs = static_cast<int>(slabs);
    j.vec4 = (a.N % 4 == 0) && (reinterpret_cast<uintptr_t>(a.w) % 16 == 0);
    j.gx1 = static_cast<unsigned>(cdiv(a.N, 64));
    j.gx2 = static_cast<unsigned>(cdiv(a.N, kWCols));
    d.first1[i] = static_cast<unsigned>(b1);
    d.first2[i] = static_cast<unsigned>(b2);
    b1 += static_cast<uint64_t>(j.gx1) * static_cast<uint64_t>(slabs);
    b2 += static_cast<uint64_t>(j.gx2) * static_cast<uint64_t>(cdiv(a.K, kWChunk));
    j.part = a.part; j.wq_packed = static_cast<uint8_t *>(a.wq_packed); j.s_w = a.s_w; j.wq_kn = a.wq_kn;
    j.mask_w = a.mask_w; j.wfrag = static_cast<uint4 *>(a.wfrag);
  }
  for (int i = n; i < kWeightJobsMax; ++i) d.job[i] = d.job[0];   // never selected: job_of_block stops at n
  for (int i = n; i <= kWeightJobsMax; ++i) {
    d.first1[i] = static_cast<unsigned>(b1);
    d.first2[i] = static_cast<unsigned>(b2);
  }
  d.n = n;
  if (b1 > 0x7FFFFFFFu || b2 > 0x7FFFFFFFu) return AQT_ERR_UNSUPPORTED;
  wabsmax_partial_group_kernel<<<static_cast<unsigned>(b1), kThreads, 0, st>>>(d);
  AQT_HIP(hipGetLastError());
  quantize_weights_group_kernel<<<static_cast<unsigned>(b2), kThreads, 0, st>>>(d, dev_status);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_unpack_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, int8_t *codes_kn,
                                 hipStream_t st) {
  unpack_weights_kernel<<<static_cast<int>(cdiv(K * N, kThreads)), kThreads, 0, st>>>(
      static_cast<const uint8_t *>(wq_packed), K, N, packed4(bits_w) ? 1 : 0, codes_kn);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
