// Forward contraction of the quantized dense layer (arxiv 2203.15952, Sec. 1:
// native integer matmul; Sec. 2.2: de-quantize by multiplying with the scales)
// for gfx950:  acc = xq . wq in int32 on the int8 matrix cores, then
// v = float(acc) * (s_x * s_w[n]) (+ bias), then none / Swish / GLU.
//
// The tuned kernel is described where it is defined; shapes it does not cover take
// a one-thread-per-output kernel with identical results.
#include <mutex>
#include <type_traits>

#include "aqt_internal.h"
#include "epilogue.h"

// Scratch of the entry point that allocates nothing (aqt_dense_fwd_q_static): the weight
// codes in MFMA-fragment order, K * N bytes.  Every GPU the library runs on holds its own
// copy of this array at its own address until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) uint8_t scratch[AQT_STATIC_SCRATCH_BYTES];

namespace aqt {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;

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

// max|y| as an unsigned maximum over bit patterns (non-negative floats order like
// their bits; NaN and Inf come out on top, which is how the consumer learns of them).
// The word only grows, so a stale read can only cause a redundant atomic.
__device__ __forceinline__ void note_absmax(uint32_t *y_absmax, uint32_t bits) {
  if (bits > *reinterpret_cast<volatile uint32_t *>(y_absmax)) atomicMax(y_absmax, bits);
}

__global__ void zero_word_kernel(uint32_t *p) {
  if (threadIdx.x == 0) *p = 0u;
}

__global__ __launch_bounds__(kThreads) void dense_fwd_general_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_x, const uint8_t *__restrict__ wq,
    const float *__restrict__ s_w, int64_t M, int64_t K, int64_t N, int packed,
    const float *__restrict__ bias, int epilogue, float *__restrict__ y, int32_t *__restrict__ acc_out,
    uint32_t *__restrict__ y_absmax) {
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
  if (y_absmax) note_absmax(y_absmax, __float_as_uint(out) & 0x7FFFFFFFu);
}

// ---- tuned MFMA kernel --------------------------------------------------------------
// What bounds this kernel on gfx950 is operand delivery, not the matrix cores: an
// int8 32x32x32 MFMA eats 2 KB of operands per 32 cycles, LDS delivers about 64
// bytes per clock and CU for 16-byte reads, and the K=512 layers are bound by
// writing their float32 output anyway.  Hence:
//   * The weights never touch LDS.  A small pre-kernel rewrites the forward weight
//     operand ([N][K] int8 or [N][K/2] packed int4) into MFMA-fragment order --
//     expanding int4 nibbles c to the byte 16*c on the way (a shift and a mask, the
//     sign comes for free) -- and every wavefront pulls its 1 KB fragments straight
//     from L2 with one coalesced load each, one stage ahead, into registers that
//     are refilled in place.  The accumulator is shifted back by 4 at the end,
//     which is exact because every partial sum is a multiple of 16.
//   * The activations (the HBM stream) go global -> registers (two alternating
//     sets, a full stage in flight) -> LDS (two slots, 128-byte rows, 16-byte chunks
//     XOR-swizzled with the row) -> fragments refilled in place.
//   * Workgroup = 2 x 2 wavefronts, tile (64*TM) x (64*TN) with TM < TN so that LDS
//     reads per MFMA are 1/TN KB; 128 fan-in bytes per stage = 4 MFMA steps; one
//     barrier per stage; two workgroups per CU.  All non-MFMA work is cut into
//     pieces slotted between MFMAs; the loop body is branch-free (loads past the
//     end are clamped to the last stage).
constexpr int kBK = 128;     // fan-in bytes per stage
constexpr int kKK = 4;       // MFMA steps (32 fan-in each) per stage

#define AQT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int waitcnt_imm(int vm, int lgkm) {   // s_waitcnt immediate, gfx9 layout
  return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 0xF) << 8);
}

// int4 -> int8 (times 16): eight nibbles of one dword, fan-in order c0..c7, become
// the two dwords {16c0,16c1,16c2,16c3} and {16c4,..,16c7}.
__device__ __forceinline__ void unpack8(uint32_t w, uint32_t &d0, uint32_t &d1) {
  const uint32_t lo = (w << 4) & 0xF0F0F0F0u;  // bytes: c0 c2 c4 c6 (each times 16)
  const uint32_t hi = w & 0xF0F0F0F0u;         // bytes: c1 c3 c5 c7
  // v_perm_b32 picks bytes out of {hi (selectors 4..7), lo (selectors 0..3)}
  d0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);  // lo.b0 hi.b0 lo.b1 hi.b1
  d1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);  // lo.b2 hi.b2 lo.b3 hi.b3
}

// Forward weight operand -> MFMA-fragment order.  Fragment (nb, ks) covers channels
// 32*nb .. +31 and fan-in 32*ks .. +31; inside it lane (lk*32 + lr) owns the 16
// consecutive fan-in positions 32*ks + 16*lk .. +15 of channel 32*nb + lr, i.e.
// what that lane feeds to v_mfma_i32_32x32x32_i8.  Fragments are ordered [nb][ks].
__global__ __launch_bounds__(kThreads) void weights_to_frag_kernel(const uint8_t *__restrict__ wq, int K, int N,
                                                                   int packed, v4i *__restrict__ out) {
  const int64_t pieces = static_cast<int64_t>(N) * (K / 16);
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  const int ksteps = K / 32;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < pieces; i += stride) {
    const int lane = static_cast<int>(i & 63);
    const int64_t frag = i >> 6;
    const int ks = static_cast<int>(frag % ksteps), nb = static_cast<int>(frag / ksteps);
    const int n = 32 * nb + (lane & 31), k = 32 * ks + 16 * (lane >> 5);
    v4i o;
    if (packed) {
      const uint2 w = *reinterpret_cast<const uint2 *>(wq + static_cast<int64_t>(n) * (K >> 1) + (k >> 1));
      uint32_t d0, d1;
      unpack8(w.x, d0, d1); o.x = d0; o.y = d1;
      unpack8(w.y, d0, d1); o.z = d0; o.w = d1;
    } else {
      o = *reinterpret_cast<const v4i *>(wq + static_cast<int64_t>(n) * K + k);
    }
    out[i] = o;
  }
}

template <int TM, int TN, bool SHIFT4, int EPI>
__global__ __launch_bounds__(kThreads, 2) void dense_fwd_mfma_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_x, const v4i *__restrict__ wfrag,
    const float *__restrict__ s_w, int M, int K, int N, const float *__restrict__ bias,
    float *__restrict__ y, int32_t *__restrict__ acc_out, uint32_t *__restrict__ y_absmax, int tiles_m,
    int tiles_n) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int NA = BM * (kBK / 16) / kThreads;   // 16-byte pieces of activations per thread per stage
  __shared__ __attribute__((aligned(1024))) uint8_t sA0[BM * kBK], sA1[BM * kBK];

  // Workgroup -> tile, row-major over (row tile, column tile).  Consecutive workgroup
  // ids land on different XCDs, so the column tiles of one row tile run at the same
  // time on different L2s and each fetches the activation tile itself; measured, that
  // costs less than what remapping ids to one contiguous run of tiles per XCD loses
  // on the output side (the tiles in flight then write to eight distant regions).
  (void)tiles_m;
  const int id = blockIdx.x;
  const int bm = id / tiles_n, bn = id - bm * tiles_n;
  // A ragged last row tile is shifted up to end at row M: it recomputes a few rows
  // of its neighbour (same values, same addresses) instead of predicating.
  const int m0 = min(bm * BM, M - BM);

  const int t = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6), lane = t & 63;   // wave index is uniform
  const int wm = wave >> 1, wn = wave & 1;
  const int lr = lane & 31, lk = lane >> 5;

  // Tile-local column block cb (32 columns) -> output channel of its first column.
  // GLU tiles pair value and gate blocks: even blocks are values, odd blocks gates.
  auto chan_of_block = [&](int cb) -> int {
    if (EPI == AQT_EPI_GLU) return ((cb & 1) ? (N >> 1) : 0) + bn * (BN / 2) + (cb >> 1) * 32;
    return bn * BN + cb * 32;
  };

  // ---- activations: global -> registers -> LDS ----
  v4i ra[2][NA];
  const char *a_base = reinterpret_cast<const char *>(xq + static_cast<int64_t>(m0) * K);
  const uint32_t ga0 = static_cast<uint32_t>((t >> 3) * K + (t & 7) * 16);   // piece i: + i * 32 rows
  const uint32_t ga_step = static_cast<uint32_t>(32 * K);
  const int rowa = t >> 3;
  const int offa0 = rowa * kBK + (((t & 7) ^ (rowa & 7)) << 4);             // + i * 32 rows keeps row & 7
  auto load_a = [&](int set, int k0) {
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[set][i] = *reinterpret_cast<const v4i *>(a_base + k0 + ga0 + i * ga_step);
  };
  auto store_a = [&](int set, int i, uint8_t *slot) {
    *reinterpret_cast<v4i *>(slot + offa0 + i * 32 * kBK) = ra[set][i];
  };
  // fragments of the activations: row lr of row tile i, 16-byte chunk (2*kk + lk) ^ (lr & 7)
  const int a_row = (wm * 32 * TM + lr) * kBK;
  v4i fa[TM];
  auto read_a = [&](const uint8_t *slot, int kk, int i) {
    fa[i] = *reinterpret_cast<const v4i *>(slot + a_row + i * 32 * kBK + (((2 * kk + lk) ^ (lr & 7)) << 4));
  };

  // ---- weights: fragments straight from L2 ----
  const int ksteps = K / 32;
  const v4i *b_blk[TN];   // uniform: fragment row of column block j
#pragma unroll
  for (int j = 0; j < TN; ++j)
    b_blk[j] = wfrag + static_cast<int64_t>(chan_of_block(wn * TN + j) / 32) * ksteps * 64;
  v4i fb[kKK][TN];
  auto load_b = [&](int kk, int j, int stage) { fb[kk][j] = (b_blk[j] + (stage * kKK + kk) * 64)[lane]; };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int NS = K / kBK;
  auto stage_idx = [&](int s) { return s < NS - 1 ? s : NS - 1; };

  // ---- prologue ----
  load_a(0, 0);
#pragma unroll
  for (int kk = 0; kk < kKK; ++kk)
#pragma unroll
    for (int j = 0; j < TN; ++j) load_b(kk, j, 0);
#pragma unroll
  for (int i = 0; i < NA; ++i) store_a(0, i, sA0);
  load_a(1, stage_idx(1) * kBK);
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int i = 0; i < TM; ++i) read_a(sA0, 0, i);

  // One stage; PAR = s % 2 is a compile-time constant (register sets, LDS slots).
  // MFMA q = i*TN + j of a step: row tile i uses its activation fragment in TN
  // consecutive MFMAs and is refilled right after; weight fragment j is last used
  // by row tile TM-1 and is refilled (for the next stage, same step) right after.
  auto stage = [&](auto par, int s) {
    constexpr int PAR = decltype(par)::value;
    uint8_t *cur = PAR ? sA1 : sA0;
    uint8_t *nxt = PAR ? sA0 : sA1;
    const int s1 = stage_idx(s + 1);
    load_a(PAR, stage_idx(s + 2) * kBK);   // set PAR was written to LDS one stage ago
    AQT_SCHED_FENCE();
#pragma unroll
    for (int kk = 0; kk < kKK; ++kk) {
      if (kk == kKK - 1) {
        // next stage fully staged by everybody before its first fragments are read
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
        __builtin_amdgcn_s_barrier();
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[kk][j], acc[i][j], 0, 0, 0);
          if (j & 1) {
            AQT_SCHED_FENCE();
            if (i == TM - 1) { load_b(kk, j - 1, s1); load_b(kk, j, s1); }
            // stage s + 1 into the other slot during steps 0 and 1
            if (kk < 2) {
              constexpr int PER = (NA + 2 * TM * TN / 2 - 1) / (2 * TM * TN / 2);
              const int slot_no = (kk * TM + i) * (TN / 2) + (j >> 1);
#pragma unroll
              for (int c = slot_no * PER; c < (slot_no + 1) * PER && c < NA; ++c) store_a(PAR ^ 1, c, nxt);
            }
            AQT_SCHED_FENCE();
          }
        }
        // row tile i done for this step: refill its fragment for the next step
        if (kk < kKK - 1) read_a(cur, kk + 1, i);
        else read_a(nxt, 0, i);
        AQT_SCHED_FENCE();
      }
    }
  };

  int s = 0;
  for (; s + 1 < NS; s += 2) {
    stage(std::integral_constant<int, 0>{}, s);
    stage(std::integral_constant<int, 1>{}, s + 1);
  }
  if (s < NS) stage(std::integral_constant<int, 0>{}, s);

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
      const int lane_off = row_l * N + chan_of_block(wn * TN + j) + lr;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int a0 = SHIFT4 ? (acc[i][j][r] >> 4) : acc[i][j][r];
          abase[(i * 32 + 8 * (r >> 2) + (r & 3)) * N + lane_off] = a0;
        }
    }
  }
  float *ybase = y + static_cast<int64_t>(m0) * out_cols;
  uint32_t amax = 0u;   // running max|out| of this lane, as a bit pattern
#pragma unroll
  for (int j = 0; j < TN; j += JS) {
    const int n_a = chan_of_block(wn * TN + j) + lr;   // for GLU: the value channel = output column
    const float sc_a = sx * s_w[n_a];
    const float bias_a = bias ? bias[n_a] : 0.0f;
    float sc_b = 0.0f, bias_b = 0.0f;
    if (EPI == AQT_EPI_GLU) {
      const int n_b = chan_of_block(wn * TN + j + 1) + lr;
      sc_b = sx * s_w[n_b];
      bias_b = bias ? bias[n_b] : 0.0f;
    }
    const int lane_off = row_l * out_cols + n_a;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int a0 = SHIFT4 ? (acc[i][j][r] >> 4) : acc[i][j][r];
        const float v = dequant_f32(a0, sc_a) + bias_a;   // adding a zero bias changes nothing
        float out;
        if (EPI == AQT_EPI_NONE) {
          out = v;
        } else if (EPI == AQT_EPI_SWISH) {
          out = swish_f32(v);
        } else {
          const int a1 = SHIFT4 ? (acc[i][j + (JS - 1)][r] >> 4) : acc[i][j + (JS - 1)][r];
          const float g = dequant_f32(a1, sc_b) + bias_b;
          out = v * sigmoid_f32(g);
        }
        // written once, read by another kernel much later: stream it past the caches
        __builtin_nontemporal_store(out, ybase + (i * 32 + 8 * (r >> 2) + (r & 3)) * out_cols + lane_off);
        amax = max(amax, __float_as_uint(out) & 0x7FFFFFFFu);
      }
    }
  }
  if (y_absmax) {   // uniform: one atomic per wavefront, and only if it can raise the word
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = max(amax, static_cast<uint32_t>(__shfl_xor(static_cast<int>(amax), off)));
    if (lane == 0) note_absmax(y_absmax, amax);
  }
}

template <int TM, int TN, bool SHIFT4, int EPI>
aqt_status launch_mfma(const int8_t *xq, const float *s_x, const v4i *wfrag, const float *s_w, int64_t M,
                       int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out, uint32_t *y_absmax,
                       hipStream_t st) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  auto kern = dense_fwd_mfma_kernel<TM, TN, SHIFT4, EPI>;
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_n = static_cast<int>(N / BN);
  kern<<<tiles_m * tiles_n, kThreads, 0, st>>>(xq, s_x, wfrag, s_w, static_cast<int>(M), static_cast<int>(K),
                                               static_cast<int>(N), bias, y, acc_out, y_absmax, tiles_m, tiles_n);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

template <int TM, int TN, bool SHIFT4>
aqt_status launch_mfma_epi(int epilogue, const int8_t *xq, const float *s_x, const v4i *wfrag, const float *s_w,
                           int64_t M, int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out,
                           uint32_t *y_absmax, hipStream_t st) {
  switch (epilogue) {
    case AQT_EPI_NONE: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_NONE>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st);
    case AQT_EPI_SWISH: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_SWISH>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st);
    default: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_GLU>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st);
  }
}

}  // namespace

size_t fwd_q_workspace_bytes(int64_t K, int64_t N) { return align_up(static_cast<size_t>(K) * N, 256); }

// Device address of `scratch` on the current device, looked up once per device.
aqt_status static_scratch_address(void **out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void *addr[kMaxDevices] = {};
  int dev = 0;
  AQT_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return AQT_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *p = nullptr;
    AQT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return AQT_ERR_HIP;
    addr[dev] = p;
  }
  *out = addr[dev];
  return AQT_OK;
}

aqt_status launch_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                              int64_t M, int64_t K, int64_t N, int bits_w, const float *bias, int epilogue,
                              float *y, int32_t *acc_out, uint32_t *y_absmax, void *ws, hipStream_t st) {
  const bool packed = packed4(bits_w);
  if (y_absmax) {
    zero_word_kernel<<<1, 64, 0, st>>>(y_absmax);
    AQT_HIP(hipGetLastError());
  }
  const bool aligned = (reinterpret_cast<uintptr_t>(xq) % 16 == 0) &&
                       (reinterpret_cast<uintptr_t>(wq_packed) % 16 == 0) && ws &&
                       (reinterpret_cast<uintptr_t>(ws) % 16 == 0);
  const bool sizes_fit = M < (int64_t(1) << 31) / (K > N ? K : N);  // 32-bit tile arithmetic inside
  if (aligned && sizes_fit && K % kBK == 0 && M >= 128) {
    // The column tile must divide N (N/2 for GLU, whose tile holds value and gate halves).
    // 128 x 256 tiles once there are enough of them to fill the chip, else 128 x 128.
    const int64_t nn = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
    const int64_t unit_wide = (epilogue == AQT_EPI_GLU) ? 128 : 256;
    const int64_t unit = (epilogue == AQT_EPI_GLU) ? 64 : 128;
    if (nn % unit == 0) {
      v4i *wfrag = static_cast<v4i *>(ws);
      const int64_t pieces = N * (K / 16);
      int g = static_cast<int>(cdiv(pieces, kThreads));
      if (g > 2048) g = 2048;
      weights_to_frag_kernel<<<g, kThreads, 0, st>>>(static_cast<const uint8_t *>(wq_packed), static_cast<int>(K),
                                                     static_cast<int>(N), packed ? 1 : 0, wfrag);
      AQT_HIP(hipGetLastError());
      const bool wide = (nn % unit_wide == 0) && cdiv(M, 128) * (N / 256) >= 512;
      if (wide) {
        return packed ? launch_mfma_epi<2, 4, true>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st)
                      : launch_mfma_epi<2, 4, false>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st);
      }
      return packed ? launch_mfma_epi<2, 2, true>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st)
                    : launch_mfma_epi<2, 2, false>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, st);
    }
  }
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  dense_fwd_general_kernel<<<static_cast<int>(cdiv(M * ncols, kThreads)), kThreads, 0, st>>>(
      xq, s_x, static_cast<const uint8_t *>(wq_packed), s_w, M, K, N, packed ? 1 : 0, bias, epilogue, y,
      acc_out, y_absmax);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
