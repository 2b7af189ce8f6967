// Straight-through backward of the quantized dense layer (arxiv 2203.15952:
// Fig. 2 holds the scale constant with stop_gradient; the rounding is passed
// straight through), for gfx950:
//   dx[m,k]  = mask_x[m,k] * sum_n (dy[m,n] * s_w[n]) * wq[k,n]
//   dw[k,n]  = mask_w[k,n] * s_x * sum_m xq[m,k] * dy[m,n]
//   dbias[n] = sum_m dy[m,n]
// A NULL mask stands for "the group's scale is non-zero".
//
// Both contractions pair small integer codes with float32 gradients.  Codes
// (|c| <= 127) are exact in bf16; the float operand a is split into
// hi = bf16(a) and lo = bf16(a - hi) (round to nearest even), which keeps 16
// significant bits (relative error <= 2^-16 per term), and two
// v_mfma_f32_32x32x16_bf16 passes accumulate code*hi + code*lo in float32.
// Every product is exact in float32, so the only other error is the float32
// accumulation itself.
#include "aqt_internal.h"

namespace aqt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;

__device__ __forceinline__ bool mask_bit(const uint32_t *__restrict__ mask, int64_t i) {
  return (mask[i >> 5] >> (i & 31)) & 1u;
}

// Two floats -> packed bf16 pair (round to nearest even).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  v2f f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

// hi/lo split of two floats: hi = bf16(a), lo = bf16(a - float(hi)).
__device__ __forceinline__ void split_bf16(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = pack_bf16(a, b);
  const float ha = __uint_as_float(hi << 16), hb = __uint_as_float(hi & 0xFFFF0000u);
  lo = pack_bf16(a - ha, b - hb);
}

__device__ __forceinline__ v16f mfma_bf16(v4i a, v4i b, v16f c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
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

// int8 codes [K,N] -> bf16 [K,N] (exact), the dX kernel's second operand.
__global__ __launch_bounds__(kThreads) void codes_to_bf16_kernel(const int8_t *__restrict__ codes, int64_t n4,
                                                                 uint32_t *__restrict__ out) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  const uint32_t *c4 = reinterpret_cast<const uint32_t *>(codes);
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < n4; i += stride) {
    const uint32_t w = c4[i];
    const float f0 = static_cast<float>(static_cast<int8_t>(w)), f1 = static_cast<float>(static_cast<int8_t>(w >> 8));
    const float f2 = static_cast<float>(static_cast<int8_t>(w >> 16)), f3 = static_cast<float>(static_cast<int8_t>(w >> 24));
    out[2 * i] = pack_bf16(f0, f1);
    out[2 * i + 1] = pack_bf16(f2, f3);
  }
}

// =====================================================================================
// dX = (dy * s_w) . wq^T       rows m, columns k, contraction over n
// Both operands are contraction-contiguous in memory (dy is [M,N], the bf16 codes
// are [K,N]).  Workgroup = 2 x 2 wavefronts, tile (64*TM) x (64*TN); 32 n per
// LDS stage; dy is scaled and split on its way into LDS.
// =====================================================================================
constexpr int kSN = 32;              // contraction elements per stage
constexpr int kPitch = kSN * 2 + 16; // LDS row pitch in bytes (bf16 rows of 32, padded)

template <int TM, int TN>
__global__ __launch_bounds__(kThreads) void bwd_dx_mfma_kernel(
    const float *__restrict__ dy, const uint16_t *__restrict__ wq_bf, const float *__restrict__ s_w,
    const float *__restrict__ s_x, const uint32_t *__restrict__ mask_x, int M, int K, int N,
    float *__restrict__ dx, int tiles_m, int tiles_c) {
  constexpr int BM = 64 * TM, BC = 64 * TN;
  constexpr int kStage = (2 * BM + BC) * kPitch;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  int id = blockIdx.x;
  const int total = tiles_m * tiles_c;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);  // one run of tiles per XCD
  const int bm = id / tiles_c, bc = id - bm * tiles_c;
  const int m0 = bm * BM, c0 = bc * BC;

  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;

  float4 ra[2 * TM];
  float4 rs;
  v4i rb[TN];

  auto load_global = [&](int n0) {
    rs = *reinterpret_cast<const float4 *>(s_w + n0 + (t & 7) * 4);
#pragma unroll
    for (int i = 0; i < 2 * TM; ++i) {
      const int c = t + kThreads * i;
      int row = m0 + (c >> 3);
      row = row < M ? row : M - 1;
      ra[i] = *reinterpret_cast<const float4 *>(dy + static_cast<int64_t>(row) * N + n0 + (c & 7) * 4);
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int c = t + kThreads * i;
      rb[i] = *reinterpret_cast<const v4i *>(wq_bf + static_cast<int64_t>(c0 + (c >> 2)) * N + n0 + (c & 3) * 8);
    }
  };

  auto store_lds = [&](int buf) {
    uint8_t *Ahi = lds + buf * kStage;
    uint8_t *Alo = Ahi + BM * kPitch;
    uint8_t *B = Alo + BM * kPitch;
#pragma unroll
    for (int i = 0; i < 2 * TM; ++i) {
      const int c = t + kThreads * i;
      const int off = (c >> 3) * kPitch + (c & 7) * 8;
      v2i hi, lo;
      uint32_t h, l;
      split_bf16(ra[i].x * rs.x, ra[i].y * rs.y, h, l); hi.x = h; lo.x = l;
      split_bf16(ra[i].z * rs.z, ra[i].w * rs.w, h, l); hi.y = h; lo.y = l;
      *reinterpret_cast<v2i *>(Ahi + off) = hi;
      *reinterpret_cast<v2i *>(Alo + off) = lo;
    }
#pragma unroll
    for (int i = 0; i < TN; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<v4i *>(B + (c >> 2) * kPitch + (c & 3) * 16) = rb[i];
    }
  };

  v16f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int NT = N / kSN;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int nt = 0; nt < NT; ++nt) {
    const int buf = nt & 1;
    if (nt + 1 < NT) load_global((nt + 1) * kSN);
    const uint8_t *Ahi = lds + buf * kStage + (wm * 32 * TM + lr) * kPitch + lk * 16;
    const uint8_t *Alo = Ahi + BM * kPitch;
    const uint8_t *B = lds + buf * kStage + 2 * BM * kPitch + (wn * 32 * TN + lr) * kPitch + lk * 16;
#pragma unroll
    for (int kk = 0; kk < kSN / 16; ++kk) {
      v4i ah[TM], al[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        ah[i] = *reinterpret_cast<const v4i *>(Ahi + i * 32 * kPitch + kk * 32);
        al[i] = *reinterpret_cast<const v4i *>(Alo + i * 32 * kPitch + kk * 32);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const v4i *>(B + j * 32 * kPitch + kk * 32);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = mfma_bf16(ah[i], b[j], acc[i][j]);
          acc[i][j] = mfma_bf16(al[i], b[j], acc[i][j]);
        }
    }
    if (nt + 1 < NT) store_lds(buf ^ 1);
    __syncthreads();
  }

  const bool pass_all = mask_x ? true : (s_x[0] != 0.0f);
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int k = c0 + wn * 32 * TN + j * 32 + lr;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 * TM + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        if (m >= M) continue;
        const int64_t idx = static_cast<int64_t>(m) * K + k;
        bool pass = pass_all;
        if (mask_x) pass = mask_bit(mask_x, idx);
        dx[idx] = pass ? acc[i][j][r] : 0.0f;
      }
  }
}

// =====================================================================================
// dW = s_x * xq^T . dy         rows k, columns n, contraction over m
// Neither operand is contraction-contiguous in memory, so each thread gathers a
// 4 (k or n) x 8 (m) block with coalesced row-wise loads, transposes it in
// registers and writes 16-byte, m-contiguous pieces into LDS.  Tile-local row
// index rho of the LDS images is de-interleaved, column 4*g + b lives in row
// b*(B/4) + g, so that the 64 lanes of a wavefront write 64 consecutive rows.
// The contraction is split over row slabs of M; each workgroup writes a float32
// partial tile and a second kernel folds the slabs in a fixed order (run-to-run
// reproducible), applies s_x and the mask.
// =====================================================================================
template <int T>  // tile is (64*T) x (64*T); SM = 128/T rows of m per stage
__global__ __launch_bounds__(kThreads) void bwd_dw_mfma_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ dy, int M, int K, int N, int m_per_slab,
    float *__restrict__ partial, int tiles_r, int tiles_c) {
  constexpr int BT = 64 * T;             // tile edge (k rows, n columns)
  constexpr int SM = 128 / T;            // m per stage: 32 (T=4) or 64 (T=2)
  constexpr int G = BT / 4;              // 4-column groups per tile edge
  constexpr int kP = SM * 2 + 16;        // LDS row pitch in bytes
  constexpr int kStage = 3 * BT * kP;    // codes, dy hi, dy lo
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const int tiles = tiles_r * tiles_c;
  const int slab = blockIdx.x / tiles;
  const int tile = blockIdx.x - slab * tiles;
  const int br = tile / tiles_c, bc = tile - br * tiles_c;
  const int r0 = br * BT, c0 = bc * BT;
  const int m_begin = slab * m_per_slab;
  const int m_end = min(M, m_begin + m_per_slab);

  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;
  const int g = t % G, mg = t / G;       // this thread's column group and m group (8 rows of m)

  uint32_t rx[8];
  float4 ry[8];

  auto load_global = [&](int mbase) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int m = mbase + mg * 8 + i;
      if (m < m_end) {
        rx[i] = *reinterpret_cast<const uint32_t *>(xq + static_cast<int64_t>(m) * K + r0 + 4 * g);
        ry[i] = *reinterpret_cast<const float4 *>(dy + static_cast<int64_t>(m) * N + c0 + 4 * g);
      } else {
        rx[i] = 0;
        ry[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };

  auto store_lds = [&](int buf) {
    uint8_t *A = lds + buf * kStage;
    uint8_t *Bhi = A + BT * kP;
    uint8_t *Blo = Bhi + BT * kP;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      // codes: byte b of the eight dwords -> eight bf16 along m
      float f[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = static_cast<float>(static_cast<int8_t>(rx[i] >> (8 * b)));
      v4i a;
      a.x = pack_bf16(f[0], f[1]); a.y = pack_bf16(f[2], f[3]);
      a.z = pack_bf16(f[4], f[5]); a.w = pack_bf16(f[6], f[7]);
      const int row = b * G + g;
      *reinterpret_cast<v4i *>(A + row * kP + mg * 16) = a;
      // gradients: component b of the eight float4 -> hi/lo bf16 along m
      float y[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = b == 0 ? ry[i].x : (b == 1 ? ry[i].y : (b == 2 ? ry[i].z : ry[i].w));
      v4i hi, lo;
      uint32_t h, l;
      split_bf16(y[0], y[1], h, l); hi.x = h; lo.x = l;
      split_bf16(y[2], y[3], h, l); hi.y = h; lo.y = l;
      split_bf16(y[4], y[5], h, l); hi.z = h; lo.z = l;
      split_bf16(y[6], y[7], h, l); hi.w = h; lo.w = l;
      *reinterpret_cast<v4i *>(Bhi + row * kP + mg * 16) = hi;
      *reinterpret_cast<v4i *>(Blo + row * kP + mg * 16) = lo;
    }
  };

  v16f acc[T][T];
#pragma unroll
  for (int i = 0; i < T; ++i)
#pragma unroll
    for (int j = 0; j < T; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int stages = (m_end - m_begin + SM - 1) / SM;
  if (stages > 0) {
    load_global(m_begin);
    store_lds(0);
  }
  __syncthreads();
  for (int s = 0; s < stages; ++s) {
    const int buf = s & 1;
    if (s + 1 < stages) load_global(m_begin + (s + 1) * SM);
    const uint8_t *A = lds + buf * kStage + (wm * 32 * T + lr) * kP + lk * 16;
    const uint8_t *Bhi = lds + buf * kStage + BT * kP + (wn * 32 * T + lr) * kP + lk * 16;
    const uint8_t *Blo = Bhi + BT * kP;
#pragma unroll
    for (int kk = 0; kk < SM / 16; ++kk) {
      v4i a[T], bh[T], bl[T];
#pragma unroll
      for (int i = 0; i < T; ++i) a[i] = *reinterpret_cast<const v4i *>(A + i * 32 * kP + kk * 32);
#pragma unroll
      for (int j = 0; j < T; ++j) {
        bh[j] = *reinterpret_cast<const v4i *>(Bhi + j * 32 * kP + kk * 32);
        bl[j] = *reinterpret_cast<const v4i *>(Blo + j * 32 * kP + kk * 32);
      }
#pragma unroll
      for (int i = 0; i < T; ++i)
#pragma unroll
        for (int j = 0; j < T; ++j) {
          acc[i][j] = mfma_bf16(a[i], bh[j], acc[i][j]);
          acc[i][j] = mfma_bf16(a[i], bl[j], acc[i][j]);
        }
    }
    if (s + 1 < stages) store_lds(buf ^ 1);
    __syncthreads();
  }

  float *out = partial + static_cast<int64_t>(slab) * K * N;
#pragma unroll
  for (int j = 0; j < T; ++j) {
    const int rho_c = wn * 32 * T + j * 32 + lr;
    const int n = c0 + 4 * (rho_c % G) + rho_c / G;
#pragma unroll
    for (int i = 0; i < T; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rho_r = wm * 32 * T + i * 32 + 8 * (r >> 2) + 4 * lk + (r & 3);
        const int k = r0 + 4 * (rho_r % G) + rho_r / G;
        out[static_cast<int64_t>(k) * N + n] = acc[i][j][r];
      }
  }
}

// Fold the slabs in order, scale by s_x, apply the mask.
__global__ __launch_bounds__(kThreads) void bwd_dw_fold_kernel(const float *__restrict__ partial, int slabs,
                                                               int64_t KN, int64_t N, const float *__restrict__ s_x,
                                                               const float *__restrict__ s_w,
                                                               const uint32_t *__restrict__ mask_w,
                                                               float *__restrict__ dw) {
  const int64_t i4 = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t i = i4 * 4;
  if (i >= KN) return;
  float4 s = *reinterpret_cast<const float4 *>(partial + i);
  for (int j = 1; j < slabs; ++j) {
    const float4 p = *reinterpret_cast<const float4 *>(partial + static_cast<int64_t>(j) * KN + i);
    s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
  }
  const float sx = s_x[0];
  float v[4] = {sx * s.x, sx * s.y, sx * s.z, sx * s.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int64_t idx = i + e;
    const bool pass = mask_w ? mask_bit(mask_w, idx) : (s_w[idx % N] != 0.0f);
    if (!pass) v[e] = 0.0f;
  }
  *reinterpret_cast<float4 *>(dw + i) = make_float4(v[0], v[1], v[2], v[3]);
}

struct BwdPlan {
  bool dx_mfma, dw_mfma;
  int dx_t;        // 4 or 2: tile edge 256 or 128
  int dw_t;
  int slabs;
  int m_per_slab;
  size_t off_bf, off_part, off_bias, total;
};

BwdPlan plan_bwd(int64_t M, int64_t K, int64_t N) {
  BwdPlan p{};
  const bool fits32 = M < (int64_t(1) << 31) / (K > N ? K : N);
  // dX: columns are K, contraction N in stages of 32
  p.dx_mfma = fits32 && (N % kSN == 0) && (K % 128 == 0);
  p.dx_t = (K % 256 == 0 && cdiv(M, 256) * (K / 256) >= 512) ? 4 : 2;
  // dW: tiles over K x N, slabs over M
  p.dw_mfma = fits32 && (K % 128 == 0) && (N % 128 == 0);
  p.dw_t = (K % 256 == 0 && N % 256 == 0 && (K / 256) * (N / 256) >= 16) ? 4 : 2;
  const int edge = 64 * p.dw_t;
  const int64_t tiles = (K / edge) * (N / edge);
  int64_t slabs = p.dw_mfma ? cdiv(512, tiles) : 1;
  if (slabs > 64) slabs = 64;
  int64_t per = cdiv(M, slabs);
  per = cdiv(per, 64) * 64;            // whole stages
  slabs = cdiv(M, per);
  p.slabs = static_cast<int>(slabs);
  p.m_per_slab = static_cast<int>(per);
  size_t off = 0;
  p.off_bf = off;   off += align_up(static_cast<size_t>(K) * N * 2, 256);
  p.off_part = off; off += align_up(static_cast<size_t>(p.slabs) * K * N * 4, 256);
  p.off_bias = off; off += align_up(static_cast<size_t>(kBiasSlabs) * N * sizeof(double), 256);
  p.total = off;
  return p;
}

template <int TM, int TN>
aqt_status launch_dx(const float *dy, const uint16_t *wq_bf, const aqt_saved *sv, int64_t M, int64_t K, int64_t N,
                     float *dx, hipStream_t st) {
  constexpr int BM = 64 * TM, BC = 64 * TN;
  constexpr int smem = 2 * (2 * BM + BC) * kPitch;
  auto kern = bwd_dx_mfma_kernel<TM, TN>;
  static bool attr_set = false;
  if (!attr_set) {
    AQT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    attr_set = true;
  }
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_c = static_cast<int>(K / BC);
  kern<<<tiles_m * tiles_c, kThreads, smem, st>>>(dy, wq_bf, sv->s_w, sv->s_x, sv->mask_x, static_cast<int>(M),
                                                  static_cast<int>(K), static_cast<int>(N), dx, tiles_m, tiles_c);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

template <int T>
aqt_status launch_dw(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N, const BwdPlan &p,
                     float *partial, hipStream_t st) {
  constexpr int BT = 64 * T, SM = 128 / T;
  constexpr int smem = 2 * 3 * BT * (SM * 2 + 16);
  auto kern = bwd_dw_mfma_kernel<T>;
  static bool attr_set = false;
  if (!attr_set) {
    AQT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    attr_set = true;
  }
  const int tiles_r = static_cast<int>(K / BT), tiles_c = static_cast<int>(N / BT);
  kern<<<tiles_r * tiles_c * p.slabs, kThreads, smem, st>>>(sv->xq, dy, static_cast<int>(M), static_cast<int>(K),
                                                            static_cast<int>(N), p.m_per_slab, partial, tiles_r,
                                                            tiles_c);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace

size_t bwd_workspace_bytes(int64_t M, int64_t K, int64_t N) { return plan_bwd(M, K, N).total; }

aqt_status launch_dense_bwd(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N, float *dx,
                            float *dw, float *dbias, void *ws, size_t ws_bytes, hipStream_t st) {
  (void)ws_bytes;
  const BwdPlan p = plan_bwd(M, K, N);
  uint8_t *base = static_cast<uint8_t *>(ws);
  const bool dy_aligned = reinterpret_cast<uintptr_t>(dy) % 16 == 0;
  if (dx) {
    if (p.dx_mfma && dy_aligned && reinterpret_cast<uintptr_t>(sv->s_w) % 16 == 0) {
      uint16_t *wq_bf = reinterpret_cast<uint16_t *>(base + p.off_bf);
      const int64_t n4 = K * N / 4;
      int g = static_cast<int>(cdiv(n4, kThreads));
      if (g > 2048) g = 2048;
      codes_to_bf16_kernel<<<g, kThreads, 0, st>>>(sv->wq_kn, n4, reinterpret_cast<uint32_t *>(wq_bf));
      AQT_HIP(hipGetLastError());
      if (p.dx_t == 4) AQT_TRY((launch_dx<4, 4>(dy, wq_bf, sv, M, K, N, dx, st)));
      else AQT_TRY((launch_dx<2, 2>(dy, wq_bf, sv, M, K, N, dx, st)));
    } else {
      bwd_dx_general_kernel<<<static_cast<int>(cdiv(M * K, kThreads)), kThreads, 0, st>>>(
          dy, sv->wq_kn, sv->s_w, sv->s_x, sv->mask_x, M, K, N, dx);
      AQT_HIP(hipGetLastError());
    }
  }
  if (dw) {
    if (p.dw_mfma && dy_aligned && reinterpret_cast<uintptr_t>(sv->xq) % 4 == 0 &&
        reinterpret_cast<uintptr_t>(dw) % 16 == 0) {
      float *partial = reinterpret_cast<float *>(base + p.off_part);
      if (p.dw_t == 4) AQT_TRY(launch_dw<4>(dy, sv, M, K, N, p, partial, st));
      else AQT_TRY(launch_dw<2>(dy, sv, M, K, N, p, partial, st));
      bwd_dw_fold_kernel<<<static_cast<int>(cdiv(K * N / 4, kThreads)), kThreads, 0, st>>>(
          partial, p.slabs, K * N, N, sv->s_x, sv->s_w, sv->mask_w, dw);
      AQT_HIP(hipGetLastError());
    } else {
      bwd_dw_general_kernel<<<static_cast<int>(cdiv(K * N, kThreads)), kThreads, 0, st>>>(
          dy, sv->xq, sv->s_x, sv->s_w, sv->mask_w, M, K, N, dw);
      AQT_HIP(hipGetLastError());
    }
  }
  if (dbias) {
    double *part = reinterpret_cast<double *>(base + p.off_bias);
    dim3 grid(static_cast<unsigned>(cdiv(N, 64)), kBiasSlabs);
    bwd_dbias_partial_kernel<<<grid, kThreads, 0, st>>>(dy, M, N, part);
    AQT_HIP(hipGetLastError());
    bwd_dbias_fold_kernel<<<static_cast<int>(cdiv(N, kThreads)), kThreads, 0, st>>>(part, N, dbias);
    AQT_HIP(hipGetLastError());
  }
  return AQT_OK;
}

}  // namespace aqt
