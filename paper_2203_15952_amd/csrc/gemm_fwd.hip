// Forward contraction of the quantized dense layer (arxiv 2203.15952, Sec. 1:
// native integer matmul; Sec. 2.2: de-quantize by multiplying with the scales)
// for gfx950:  acc = xq . wq in int32 on the int8 matrix cores, then
// v = float(acc) * (s_x * s_w[n]) (+ bias), then none / Swish / GLU.
//
// Tuned kernel: a workgroup of four wavefronts (2 x 2) owns a BM x BN output tile;
// each wavefront owns TM x TN tiles of 32 x 32 driven by v_mfma_i32_32x32x32_i8.
// Both operands are fan-in contiguous (xq is [M,K]; the weight operand is [N][K]
// or [N][K/2] packed), are staged through LDS in 64-byte K slices with register
// prefetch of the next slice, and int4 weights are expanded to int8 on their way
// into LDS.  The nibble c is expanded to the byte 16*c (a shift and a mask, the
// sign comes for free) and the accumulator is shifted back by 4 at the end, which
// is exact because every partial sum is a multiple of 16.
#include "aqt_internal.h"
#include "epilogue.h"

namespace aqt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBK = 64;            // bytes (= int8 codes) of fan-in per LDS stage
constexpr int kRow = kBK + 16;     // LDS row pitch: 80 B keeps 16-byte reads of 8 rows on distinct banks

// ---- general kernel: one thread per output, any shape -----------------------------
__device__ __forceinline__ int weight_code(const uint8_t *__restrict__ wq, int64_t row_bytes, int packed,
                                           int64_t n, int64_t k) {
  if (packed) {
    const uint32_t b = wq[n * row_bytes + (k >> 1)];
    const uint32_t nib = (k & 1) ? (b >> 4) : (b & 0xFu);
    return static_cast<int>(nib ^ 8u) - 8;
  }
  return static_cast<int8_t>(wq[n * row_bytes + k]);
}

__global__ __launch_bounds__(kThreads) void dense_fwd_general_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_x, const uint8_t *__restrict__ wq,
    const float *__restrict__ s_w, int64_t M, int64_t K, int64_t N, int packed,
    const float *__restrict__ bias, int epilogue, float *__restrict__ y, int32_t *__restrict__ acc_out) {
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (idx >= M * ncols) return;
  const int64_t m = idx / ncols, j = idx - m * ncols;
  const int64_t row_bytes = packed ? (K + 1) / 2 : K;
  const float sx = s_x[0];
  const int parts = (epilogue == AQT_EPI_GLU) ? 2 : 1;
  float v[2];
  for (int p = 0; p < parts; ++p) {
    const int64_t n = j + p * ncols;
    int acc = 0;
    for (int64_t k = 0; k < K; ++k) acc += static_cast<int>(xq[m * K + k]) * weight_code(wq, row_bytes, packed, n, k);
    if (acc_out) acc_out[m * N + n] = acc;
    float t = dequant_f32(acc, sx * s_w[n]);
    if (bias) t = t + bias[n];
    v[p] = t;
  }
  float out;
  if (epilogue == AQT_EPI_NONE) out = v[0];
  else if (epilogue == AQT_EPI_SWISH) out = swish_f32(v[0]);
  else out = v[0] * sigmoid_f32(v[1]);
  y[m * ncols + j] = out;
}

// ---- tuned MFMA kernel --------------------------------------------------------------
// int4 -> int8 (times 16): eight nibbles of one dword, fan-in order c0..c7, become
// the two dwords {16c0,16c1,16c2,16c3} and {16c4,..,16c7}.
__device__ __forceinline__ void unpack8(uint32_t w, uint32_t &d0, uint32_t &d1) {
  const uint32_t lo = (w << 4) & 0xF0F0F0F0u;  // bytes: c0 c2 c4 c6 (each times 16)
  const uint32_t hi = w & 0xF0F0F0F0u;         // bytes: c1 c3 c5 c7
  // v_perm_b32 picks bytes out of {hi (selectors 4..7), lo (selectors 0..3)}
  d0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);  // lo.b0 hi.b0 lo.b1 hi.b1
  d1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);  // lo.b2 hi.b2 lo.b3 hi.b3
}

template <int TM, int TN, bool PACKED, int EPI>
__global__ __launch_bounds__(kThreads, (TM * TN <= 8) ? 2 : 1) void dense_fwd_mfma_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_x, const uint8_t *__restrict__ wq,
    const float *__restrict__ s_w, int M, int K, int N, const float *__restrict__ bias,
    float *__restrict__ y, int32_t *__restrict__ acc_out, int tiles_m, int tiles_n) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int kStage = (BM + BN) * kRow;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of
  // them, each with its own L2); give each XCD a contiguous run of tiles so the
  // workgroups that share an activation tile also share an L2.
  int id = blockIdx.x;
  const int total = tiles_m * tiles_n;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int bm = id / tiles_n, bn = id - bm * tiles_n;
  // A ragged last row tile is shifted up to end at row M: it recomputes a few rows
  // of its neighbour (same values, same addresses) instead of predicating.
  const int m0 = min(bm * BM, M - BM);

  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;

  // LDS row rr of the weight tile <- output channel
  auto chan_of = [&](int rr) -> int {
    if (EPI == AQT_EPI_GLU) {
      const int blk = rr >> 5;
      return ((blk & 1) ? (N >> 1) : 0) + bn * (BN / 2) + (blk >> 1) * 32 + (rr & 31);
    }
    return bn * BN + rr;
  };

  // ---- global -> register staging ----
  v4i ra[TM];
  v4i rb[PACKED ? (TN / 2) : TN];
  const int64_t wrow = PACKED ? (K >> 1) : K;

  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int c = t + kThreads * i;
      const int row = m0 + (c >> 2);
      ra[i] = *reinterpret_cast<const v4i *>(xq + static_cast<int64_t>(row) * K + k0 + (c & 3) * 16);
    }
    if (PACKED) {
#pragma unroll
      for (int i = 0; i < TN / 2; ++i) {
        const int c = t + kThreads * i;
        const int n = chan_of(c >> 1);
        rb[i] = *reinterpret_cast<const v4i *>(wq + static_cast<int64_t>(n) * wrow + (k0 >> 1) + (c & 1) * 16);
      }
    } else {
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        const int c = t + kThreads * i;
        const int n = chan_of(c >> 2);
        rb[i] = *reinterpret_cast<const v4i *>(wq + static_cast<int64_t>(n) * wrow + k0 + (c & 3) * 16);
      }
    }
  };

  auto store_lds = [&](int buf) {
    uint8_t *A = lds + buf * kStage;
    uint8_t *B = A + BM * kRow;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int c = t + kThreads * i;
      *reinterpret_cast<v4i *>(A + (c >> 2) * kRow + (c & 3) * 16) = ra[i];
    }
    if (PACKED) {
#pragma unroll
      for (int i = 0; i < TN / 2; ++i) {
        const int c = t + kThreads * i;
        v4i lo, hi;
        uint32_t d0, d1;
        unpack8(static_cast<uint32_t>(rb[i].x), d0, d1); lo.x = d0; lo.y = d1;
        unpack8(static_cast<uint32_t>(rb[i].y), d0, d1); lo.z = d0; lo.w = d1;
        unpack8(static_cast<uint32_t>(rb[i].z), d0, d1); hi.x = d0; hi.y = d1;
        unpack8(static_cast<uint32_t>(rb[i].w), d0, d1); hi.z = d0; hi.w = d1;
        uint8_t *dst = B + (c >> 1) * kRow + (c & 1) * 32;
        *reinterpret_cast<v4i *>(dst) = lo;
        *reinterpret_cast<v4i *>(dst + 16) = hi;
      }
    } else {
#pragma unroll
      for (int i = 0; i < TN; ++i) {
        const int c = t + kThreads * i;
        *reinterpret_cast<v4i *>(B + (c >> 2) * kRow + (c & 3) * 16) = rb[i];
      }
    }
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int KT = K / kBK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) load_global((kt + 1) * kBK);
    const uint8_t *A = lds + buf * kStage + (wm * 32 * TM + lr) * kRow + lk * 16;
    const uint8_t *B = lds + buf * kStage + BM * kRow + (wn * 32 * TN + lr) * kRow + lk * 16;
#pragma unroll
    for (int kk = 0; kk < kBK / 32; ++kk) {
      v4i a[TM], b[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const v4i *>(A + i * 32 * kRow + kk * 32);
#pragma unroll
      for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const v4i *>(B + j * 32 * kRow + kk * 32);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: registers -> HBM ----
  // Lane holds output column (lane % 32) of each 32 x 32 tile; register r holds
  // row 8*(r/4) + 4*(lane/32) + r%4.  32 lanes write 128 contiguous bytes.
  // Addresses are a uniform tile base plus one 32-bit lane offset; row and tile
  // steps are compile-time multiples of the row length folded into the base.
  const float sx = s_x[0];
  const int out_cols = (EPI == AQT_EPI_GLU) ? (N >> 1) : N;
  constexpr int JS = (EPI == AQT_EPI_GLU) ? 2 : 1;
  const int row_l = wm * 32 * TM + 4 * lk;
  if (acc_out) {
    int32_t *abase = acc_out + static_cast<int64_t>(m0) * N;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int lane_off = row_l * N + chan_of(wn * 32 * TN + j * 32 + lr);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int a0 = PACKED ? (acc[i][j][r] >> 4) : acc[i][j][r];
          abase[(i * 32 + 8 * (r >> 2) + (r & 3)) * N + lane_off] = a0;
        }
    }
  }
  float *ybase = y + static_cast<int64_t>(m0) * out_cols;
#pragma unroll
  for (int j = 0; j < TN; j += JS) {
    const int n_a = chan_of(wn * 32 * TN + j * 32 + lr);   // for GLU: the value channel = output column
    const float sc_a = sx * s_w[n_a];
    const float bias_a = bias ? bias[n_a] : 0.0f;
    float sc_b = 0.0f, bias_b = 0.0f;
    if (EPI == AQT_EPI_GLU) {
      const int n_b = chan_of(wn * 32 * TN + (j + 1) * 32 + lr);
      sc_b = sx * s_w[n_b];
      bias_b = bias ? bias[n_b] : 0.0f;
    }
    const int lane_off = row_l * out_cols + n_a;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int a0 = PACKED ? (acc[i][j][r] >> 4) : acc[i][j][r];
        const float v = dequant_f32(a0, sc_a) + bias_a;   // adding a zero bias changes nothing
        float out;
        if (EPI == AQT_EPI_NONE) {
          out = v;
        } else if (EPI == AQT_EPI_SWISH) {
          out = swish_f32(v);
        } else {
          const int a1 = PACKED ? (acc[i][j + (JS - 1)][r] >> 4) : acc[i][j + (JS - 1)][r];
          const float g = dequant_f32(a1, sc_b) + bias_b;
          out = v * sigmoid_f32(g);
        }
        // written once, read by another kernel much later: stream it past the caches
        __builtin_nontemporal_store(out, ybase + (i * 32 + 8 * (r >> 2) + (r & 3)) * out_cols + lane_off);
      }
    }
  }
}

template <int TM, int TN, bool PACKED, int EPI>
aqt_status launch_mfma(const int8_t *xq, const float *s_x, const void *wq, const float *s_w, int64_t M,
                       int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out, hipStream_t st) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int smem = 2 * (BM + BN) * kRow;
  auto kern = dense_fwd_mfma_kernel<TM, TN, PACKED, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    AQT_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    attr_set = true;
  }
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_n = static_cast<int>(N / BN);
  kern<<<tiles_m * tiles_n, kThreads, smem, st>>>(xq, s_x, static_cast<const uint8_t *>(wq), s_w,
                                                  static_cast<int>(M), static_cast<int>(K),
                                                  static_cast<int>(N), bias, y, acc_out, tiles_m, tiles_n);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

template <int TM, int TN, bool PACKED>
aqt_status launch_mfma_epi(int epilogue, const int8_t *xq, const float *s_x, const void *wq, const float *s_w,
                           int64_t M, int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out,
                           hipStream_t st) {
  switch (epilogue) {
    case AQT_EPI_NONE: return launch_mfma<TM, TN, PACKED, AQT_EPI_NONE>(xq, s_x, wq, s_w, M, K, N, bias, y, acc_out, st);
    case AQT_EPI_SWISH: return launch_mfma<TM, TN, PACKED, AQT_EPI_SWISH>(xq, s_x, wq, s_w, M, K, N, bias, y, acc_out, st);
    default: return launch_mfma<TM, TN, PACKED, AQT_EPI_GLU>(xq, s_x, wq, s_w, M, K, N, bias, y, acc_out, st);
  }
}

}  // namespace

aqt_status launch_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                              int64_t M, int64_t K, int64_t N, int bits_w, const float *bias, int epilogue,
                              float *y, int32_t *acc_out, hipStream_t st) {
  const bool packed = packed4(bits_w);
  const bool aligned = (reinterpret_cast<uintptr_t>(xq) % 16 == 0) &&
                       (reinterpret_cast<uintptr_t>(wq_packed) % 16 == 0);
  const bool sizes_fit = M < (int64_t(1) << 31) / (K > N ? K : N);  // 32-bit tile arithmetic inside
  if (aligned && sizes_fit && K % kBK == 0) {
    // The column tile must divide N (N/2 for GLU, whose tile holds value and gate halves).
    // 256 x 128 tiles (wavefront tile 128 x 64, two workgroups per CU so that one
    // workgroup's epilogue and staging overlap the other's MFMA work) once there
    // are enough of them to fill the chip, else 128 x 128.
    const int64_t nn = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
    const int64_t unit = (epilogue == AQT_EPI_GLU) ? 64 : 128;
    if (nn % unit == 0 && M >= 128) {
      const int64_t wide_tiles = cdiv(M, 256) * (N / 128);
      if (M >= 256 && wide_tiles >= 512) {
        return packed ? launch_mfma_epi<4, 2, true>(epilogue, xq, s_x, wq_packed, s_w, M, K, N, bias, y, acc_out, st)
                      : launch_mfma_epi<4, 2, false>(epilogue, xq, s_x, wq_packed, s_w, M, K, N, bias, y, acc_out, st);
      }
      return packed ? launch_mfma_epi<2, 2, true>(epilogue, xq, s_x, wq_packed, s_w, M, K, N, bias, y, acc_out, st)
                    : launch_mfma_epi<2, 2, false>(epilogue, xq, s_x, wq_packed, s_w, M, K, N, bias, y, acc_out, st);
    }
  }
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  dense_fwd_general_kernel<<<static_cast<int>(cdiv(M * ncols, kThreads)), kThreads, 0, st>>>(
      xq, s_x, static_cast<const uint8_t *>(wq_packed), s_w, M, K, N, packed ? 1 : 0, bias, epilogue, y,
      acc_out);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
