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

#ifdef AQT_TIMELINE
static __device__ long long g_timeline_fwd[AQT_TL_SLOTS * 8];
extern "C" int aqt_timeline_fwd(void *dst, size_t bytes) {
  return static_cast<int>(hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_timeline_fwd), bytes));
}
#endif

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
    uint32_t *__restrict__ y_absmax, float *__restrict__ dact) {
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
  if (epilogue == AQT_EPI_NONE) {
    out = v[0];
  } else if (epilogue == AQT_EPI_SWISH) {
    const float sg = sigmoid_f32(v[0]);
    out = v[0] * sg;
    if (dact) dact[m * N + j] = swish_dact_f32(v[0], sg);
  } else {
    const float sg = sigmoid_f32(v[1]);
    out = v[0] * sg;
    if (dact) {
      dact[m * N + j] = sg;
      dact[m * N + j + ncols] = glu_gate_dact_f32(v[0], sg);
    }
  }
  y[m * ncols + j] = out;
  if (y_absmax) note_absmax(y_absmax, __float_as_uint(out) & 0x7FFFFFFFu);
}

// ---- tuned MFMA kernel --------------------------------------------------------------
// What bounds this kernel on gfx950 is operand delivery into vector registers (LDS
// reads and loads from L2 share about 64 bytes per clock and CU), not the matrix
// cores: an int8 32x32x32 MFMA eats 2 KB of operands per 32 cycles.  Hence:
//   * Weights stay packed all the way into registers.  A small pre-kernel re-orders
//     the forward weight operand into MFMA-fragment order; int4 weights remain two
//     codes per byte there (half the bytes to deliver), and the wavefront expands
//     them to the byte 16*c with a shift and two masks per eight codes right before
//     use (the sign comes for free).  The accumulator is shifted back by 4 at the
//     end, exact because every partial sum is a multiple of 16.  Fragments come
//     straight from L2 with one coalesced 1 KB load each, about two stages ahead.
//   * Activations (the HBM stream) never pass through registers on their way in:
//     global_load_lds writes 16 bytes per lane directly into LDS (three slots of one
//     stage each, 128-byte rows, 16-byte chunks XOR-swizzled with the row; the swizzle
//     is applied on the global-address side because the LDS side of such a load is
//     linear in the lane id).  Fragments are read from LDS and refilled in place.
//   * Workgroup = 2 x 2 wavefronts, tile (64*TM) x (64*TN) with TM < TN; 128 fan-in
//     bytes per stage = 4 MFMA steps; one barrier per stage; two workgroups per CU.
//     All non-MFMA work is cut into pieces slotted between MFMAs; the loop body is
//     branch-free (loads past the end are clamped to the last stage).
constexpr int kBK = 128;     // fan-in bytes per stage
constexpr int kKK = 4;       // MFMA steps (32 fan-in each) per stage
constexpr int kSlots = 3;    // LDS slots, one stage of activations each

#define AQT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

constexpr int waitcnt_imm(int vm, int lgkm) {   // s_waitcnt immediate, gfx9 layout
  return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 0xF) << 8);
}

// Eight int4 codes of one dword in the fragment-ordered layout (byte b: low nibble =
// code b, high nibble = code 4 + b) -> the dwords {16c0..16c3} and {16c4..16c7}.
__device__ __forceinline__ v4i expand16(uint32_t wa, uint32_t wb) {
  v4i o;
  o.x = static_cast<int>((wa << 4) & 0xF0F0F0F0u);
  o.y = static_cast<int>(wa & 0xF0F0F0F0u);
  o.z = static_cast<int>((wb << 4) & 0xF0F0F0F0u);
  o.w = static_cast<int>(wb & 0xF0F0F0F0u);
  return o;
}

// Canonical packed dword (nibble e = code e, i.e. low nibble first) -> fragment-ordered dword.
__device__ __forceinline__ uint32_t regroup_nibbles(uint32_t w) {
  uint32_t t = 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const uint32_t lo = (w >> (4 * b)) & 0xFu, hi = (w >> (4 * (4 + b))) & 0xFu;
    t |= (lo | (hi << 4)) << (8 * b);
  }
  return t;
}

// Forward weight operand -> MFMA-fragment order.
// int8 weights: fragment (nb, ks) covers channels 32*nb .. +31 and fan-in 32*ks .. +31;
// inside it lane (lk*32 + lr) owns the 16 consecutive fan-in positions 32*ks + 16*lk ..
// +15 of channel 32*nb + lr, i.e. what that lane feeds to v_mfma_i32_32x32x32_i8.
// Fragments are ordered [nb][ks], 1 KB each.
// Packed int4 weights: a 1 KB fragment (nb, kp) covers the two steps ks = 2*kp, 2*kp + 1;
// lane (lk*32 + lr) owns two dwords per step (16 codes, regrouped for expand16), step
// 2*kp first.  Fragments are ordered [nb][kp].
__global__ __launch_bounds__(kThreads) void weights_to_frag_kernel(const uint8_t *__restrict__ wq, int K, int N,
                                                                   int packed, v4i *__restrict__ out) {
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  if (packed) {
    const int64_t pieces = static_cast<int64_t>(N) * (K / 32);
    const int kpairs = K / 64;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < pieces; i += stride) {
      const int lane = static_cast<int>(i & 63);
      const int64_t frag = i >> 6;
      const int kp = static_cast<int>(frag % kpairs), nb = static_cast<int>(frag / kpairs);
      const int n = 32 * nb + (lane & 31), k = 64 * kp + 16 * (lane >> 5);
      const uint8_t *row = wq + static_cast<int64_t>(n) * (K >> 1);
      const uint2 w0 = *reinterpret_cast<const uint2 *>(row + (k >> 1));          // step 2*kp
      const uint2 w1 = *reinterpret_cast<const uint2 *>(row + ((k + 32) >> 1));   // step 2*kp + 1
      v4i o;
      o.x = static_cast<int>(regroup_nibbles(w0.x)); o.y = static_cast<int>(regroup_nibbles(w0.y));
      o.z = static_cast<int>(regroup_nibbles(w1.x)); o.w = static_cast<int>(regroup_nibbles(w1.y));
      out[i] = o;
    }
    return;
  }
  const int64_t pieces = static_cast<int64_t>(N) * (K / 16);
  const int ksteps = K / 32;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < pieces; i += stride) {
    const int lane = static_cast<int>(i & 63);
    const int64_t frag = i >> 6;
    const int ks = static_cast<int>(frag % ksteps), nb = static_cast<int>(frag / ksteps);
    const int n = 32 * nb + (lane & 31), k = 32 * ks + 16 * (lane >> 5);
    out[i] = *reinterpret_cast<const v4i *>(wq + static_cast<int64_t>(n) * K + k);
  }
}

template <int TM, int TN, bool PACKED, int EPI>
__global__ __launch_bounds__(kThreads, 2) void dense_fwd_mfma_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ s_x, const v4i *__restrict__ wfrag,
    const float *__restrict__ s_w, int M, int K, int N, const float *__restrict__ bias,
    float *__restrict__ y, int32_t *__restrict__ acc_out, uint32_t *__restrict__ y_absmax,
    float *__restrict__ dact, int tiles_m, int tiles_n) {
  constexpr bool SHIFT4 = PACKED;
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int kSlotBytes = BM * kBK;
  constexpr int NL = BM * (kBK / 16) / kThreads;   // direct 1 KB loads per wavefront per stage
  __shared__ __attribute__((aligned(1024))) uint8_t sA[kSlots * kSlotBytes];

  // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (each with its
  // own L2).  Ids i, i + 8, i + 16, .. run on one XCD next to each other in time, so they
  // walk the column tiles of ONE row strip (its activations then come from HBM once
  // and from that L2 afterwards), while the row strips in flight stay neighbours, so
  // the output being written is one compact region.
  const int id = blockIdx.x;
  int bm, bn;
  {
    const int grp = 8 * tiles_n, full = (tiles_m / 8) * grp;
    if (id < full) {
      bm = (id / grp) * 8 + (id & 7);
      bn = (id % grp) >> 3;
    } else {
      bm = (tiles_m / 8) * 8 + (id - full) / tiles_n;
      bn = (id - full) % tiles_n;
    }
  }
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

  // ---- activations: global -> LDS, directly ----
  // Load number i of wavefront w fills the LDS bytes [(w*NL + i) KB, +1 KB) of a slot, lane l
  // the 16 bytes at l*16 in there: row r = (w*NL + i)*8 + l/8, chunk slot l%8, which holds
  // global chunk (l%8) ^ (r & 7) of that row (r & 7 == (l/8) & 7).
  const char *a_base = reinterpret_cast<const char *>(xq + static_cast<int64_t>(m0) * K);
  const uint32_t ga0 = static_cast<uint32_t>((wave * NL * 8 + (lane >> 3)) * K + (((lane & 7) ^ ((lane >> 3) & 7)) << 4));
  const uint32_t ga_step = static_cast<uint32_t>(8 * K);
  auto issue_a = [&](int slot_off, int k0) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      __builtin_amdgcn_global_load_lds(
          reinterpret_cast<const __attribute__((address_space(1))) void *>(
              reinterpret_cast<uintptr_t>(a_base + k0 + ga0 + i * ga_step)),
          reinterpret_cast<__attribute__((address_space(3))) void *>(
              static_cast<uint32_t>(reinterpret_cast<uintptr_t>(sA)) + slot_off + (wave * NL + i) * 1024),
          16, 0, 0);
  };
  // fragments of the activations: row lr of row tile i, 16-byte chunk (2*kk + lk) ^ (lr & 7)
  const int a_row = (wm * 32 * TM + lr) * kBK;
  v4i fa[TM];
  auto read_a = [&](int slot_off, int kk, int i) {
    fa[i] = *reinterpret_cast<const v4i *>(sA + slot_off + a_row + i * 32 * kBK + (((2 * kk + lk) ^ (lr & 7)) << 4));
  };

  // ---- weights: fragments straight from L2 ----
  // raw[q][j]: int8 weights: the fragment of step q of the stage in flight, refilled in
  // place for the next stage; packed weights: four pair slots = two stages, stage s lives
  // in slots 2*(s%2), 2*(s%2) + 1 and a slot is refilled for stage s + 2 as soon as its
  // second step has been expanded.  ub[kk % 2][j]: expanded fragments (packed only).
  constexpr int FR = PACKED ? kKK / 2 : kKK;   // fragments per column block and stage
  const int frags_per_blk = K / (PACKED ? 64 : 32);
  const v4i *b_blk[TN];   // uniform: fragment row of column block j
#pragma unroll
  for (int j = 0; j < TN; ++j)
    b_blk[j] = wfrag + static_cast<int64_t>(chan_of_block(wn * TN + j) / 32) * frags_per_blk * 64;
  v4i raw[4][TN];
  v4i ub[2][TN];
  auto load_raw = [&](int slot, int j, int frag_no) { raw[slot][j] = (b_blk[j] + frag_no * 64)[lane]; };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int NS = K / kBK;
  auto stage_idx = [&](int s) { return s < NS - 1 ? s : NS - 1; };

  AQT_TL_DECL;
  AQT_TL(0);
  // ---- prologue ----
  int off_cur = 0, off_nxt = kSlotBytes, off_fill = 2 * kSlotBytes;
  issue_a(off_cur, 0);
#pragma unroll
  for (int q = 0; q < FR; ++q)
#pragma unroll
    for (int j = 0; j < TN; ++j) load_raw(q, j, q);
  issue_a(off_nxt, stage_idx(1) * kBK);
  if (PACKED) {
#pragma unroll
    for (int q = 0; q < FR; ++q)
#pragma unroll
      for (int j = 0; j < TN; ++j) load_raw(FR + q, j, stage_idx(1) * FR + q);
  }
  AQT_SCHED_FENCE();
  // stage 0 (activations and weights) has landed; stage 1 may still be in flight
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(NL + (PACKED ? FR * TN : 0), 0));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int i = 0; i < TM; ++i) read_a(off_cur, 0, i);
  if (PACKED) {
#pragma unroll
    for (int j = 0; j < TN; ++j) ub[0][j] = expand16(raw[0][j].x, raw[0][j].y);
  }

  AQT_TL(1);
  // One stage; PAR = s % 2 is a compile-time constant (register slots).
  // MFMA q = i*TN + j of a step: row tile i uses its activation fragment in TN
  // consecutive MFMAs and is refilled right after.  Between MFMA pairs: packed weights
  // expand one fragment of the next step (and, when that empties a pair slot, refill it
  // for the stage after next); int8 weights refill a fragment right after its last use.
  auto stage = [&](auto par, int s) {
    constexpr int PAR = decltype(par)::value;
    const int s1 = stage_idx(s + 1), s2 = stage_idx(s + 2);
    issue_a(off_fill, s2 * kBK);   // that slot was last read one stage ago, before the barrier all have passed
    AQT_SCHED_FENCE();
#pragma unroll
    for (int kk = 0; kk < kKK; ++kk) {
      if (kk == kKK - 1) {
        // next stage's activations have landed (everything issued before this stage began has),
        // own LDS reads of the current slot are done
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(NL + (PACKED ? 2 * TN : 3 * TN), 0));
        __builtin_amdgcn_s_barrier();
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (PACKED) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], ub[kk & 1][j], acc[i][j], 0, 0, 0);
          else acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], raw[kk][j], acc[i][j], 0, 0, 0);
          if (j & 1) {
            AQT_SCHED_FENCE();
            if (PACKED) {
              const int jj = i * (TN / 2) + (j >> 1);   // one fragment of the next step per gap
              if (jj < TN) {
                // step kk + 1 lives in pair slot (kk + 1) / 2 of this stage; step 0 of the next stage in its slot 0
                constexpr int P0 = 2 * PAR, P1 = 2 * PAR + 1, Q0 = 2 * (PAR ^ 1);
                if (kk == 0) { ub[1][jj] = expand16(raw[P0][jj].z, raw[P0][jj].w); load_raw(P0, jj, s2 * FR); }
                if (kk == 1) ub[0][jj] = expand16(raw[P1][jj].x, raw[P1][jj].y);
                if (kk == 2) { ub[1][jj] = expand16(raw[P1][jj].z, raw[P1][jj].w); load_raw(P1, jj, s2 * FR + 1); }
                if (kk == 3) ub[0][jj] = expand16(raw[Q0][jj].x, raw[Q0][jj].y);
              }
            } else if (i == TM - 1) {
              load_raw(kk, j - 1, s1 * FR + kk);
              load_raw(kk, j, s1 * FR + kk);
            }
            AQT_SCHED_FENCE();
          }
        }
        // row tile i done for this step: refill its fragment for the next step
        if (kk < kKK - 1) read_a(off_cur, kk + 1, i);
        else read_a(off_nxt, 0, i);
        AQT_SCHED_FENCE();
      }
    }
    const int o = off_cur; off_cur = off_nxt; off_nxt = off_fill; off_fill = o;
  };

  int s = 0;
  for (; s + 1 < NS; s += 2) {
    stage(std::integral_constant<int, 0>{}, s);
    stage(std::integral_constant<int, 1>{}, s + 1);
  }
  if (s < NS) stage(std::integral_constant<int, 0>{}, s);
  // the clamped loads of the last stages are still writing LDS: drain them before the wavefront can end
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));
  AQT_TL(2);

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
    // the activation's derivative factors, [M,N], for the backward (when asked for)
    float *dbase = dact + static_cast<int64_t>(m0) * N;
    const int lane_off_d = row_l * N + n_a;
    const int gate_step = (EPI == AQT_EPI_GLU) ? (N >> 1) : 0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int a0 = SHIFT4 ? (acc[i][j][r] >> 4) : acc[i][j][r];
        const float v = dequant_f32(a0, sc_a) + bias_a;   // adding a zero bias changes nothing
        const int row_d = (i * 32 + 8 * (r >> 2) + (r & 3)) * N;
        float out;
        if (EPI == AQT_EPI_NONE) {
          out = v;
        } else if (EPI == AQT_EPI_SWISH) {
          const float sg = sigmoid_f32(v);
          out = v * sg;
          if (dact) __builtin_nontemporal_store(swish_dact_f32(v, sg), dbase + row_d + lane_off_d);
        } else {
          const int a1 = SHIFT4 ? (acc[i][j + (JS - 1)][r] >> 4) : acc[i][j + (JS - 1)][r];
          const float g = dequant_f32(a1, sc_b) + bias_b;
          const float sg = sigmoid_f32(g);
          out = v * sg;
          if (dact) {
            __builtin_nontemporal_store(sg, dbase + row_d + lane_off_d);
            __builtin_nontemporal_store(glu_gate_dact_f32(v, sg), dbase + row_d + lane_off_d + gate_step);
          }
        }
        // written once, read by another kernel much later: stream it past the caches
        __builtin_nontemporal_store(out, ybase + (i * 32 + 8 * (r >> 2) + (r & 3)) * out_cols + lane_off);
        amax = max(amax, __float_as_uint(out) & 0x7FFFFFFFu);
      }
    }
  }
#ifdef AQT_TIMELINE
  AQT_TL(3);
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // the stores have been acknowledged
  AQT_TL(4);
  AQT_TL_WRITE(g_timeline_fwd, bm * 65536 + bn);
#endif
  if (y_absmax) {   // uniform: one atomic per wavefront, and only if it can raise the word
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = max(amax, static_cast<uint32_t>(__shfl_xor(static_cast<int>(amax), off)));
    if (lane == 0) note_absmax(y_absmax, amax);
  }
}

template <int TM, int TN, bool SHIFT4, int EPI>
aqt_status launch_mfma(const int8_t *xq, const float *s_x, const v4i *wfrag, const float *s_w, int64_t M,
                       int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out, uint32_t *y_absmax,
                       float *dact, hipStream_t st) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  auto kern = dense_fwd_mfma_kernel<TM, TN, SHIFT4, EPI>;
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_n = static_cast<int>(N / BN);
  kern<<<tiles_m * tiles_n, kThreads, 0, st>>>(xq, s_x, wfrag, s_w, static_cast<int>(M), static_cast<int>(K),
                                               static_cast<int>(N), bias, y, acc_out, y_absmax, dact, tiles_m, tiles_n);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

template <int TM, int TN, bool SHIFT4>
aqt_status launch_mfma_epi(int epilogue, const int8_t *xq, const float *s_x, const v4i *wfrag, const float *s_w,
                           int64_t M, int64_t K, int64_t N, const float *bias, float *y, int32_t *acc_out,
                           uint32_t *y_absmax, float *dact, hipStream_t st) {
  switch (epilogue) {
    case AQT_EPI_NONE: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_NONE>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st);
    case AQT_EPI_SWISH: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_SWISH>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st);
    default: return launch_mfma<TM, TN, SHIFT4, AQT_EPI_GLU>(xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st);
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

bool fwd_q_takes_fragments(int64_t M, int64_t K, int64_t N, int epilogue) {
  const bool sizes_fit = M < (int64_t(1) << 31) / (K > N ? K : N);  // 32-bit tile arithmetic inside
  // The column tile must divide N (N/2 for GLU, whose tile holds value and gate halves).
  const int64_t nn = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  const int64_t unit = (epilogue == AQT_EPI_GLU) ? 64 : 128;
  return sizes_fit && K % kBK == 0 && M >= 128 && nn % unit == 0;
}

aqt_status launch_prepare_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, void *wprep,
                                  hipStream_t st) {
  const bool packed = packed4(bits_w);
  const int64_t pieces = N * (K / (packed ? 32 : 16));
  int g = static_cast<int>(cdiv(pieces, kThreads));
  if (g > 2048) g = 2048;
  weights_to_frag_kernel<<<g, kThreads, 0, st>>>(static_cast<const uint8_t *>(wq_packed), static_cast<int>(K),
                                                 static_cast<int>(N), packed ? 1 : 0, static_cast<v4i *>(wprep));
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

aqt_status launch_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                              int64_t M, int64_t K, int64_t N, int bits_w, const float *bias, int epilogue,
                              float *y, int32_t *acc_out, uint32_t *y_absmax, void *ws, hipStream_t st,
                              float *dact, bool ws_is_prepared, bool absmax_is_zero) {
  const bool packed = packed4(bits_w);
  if (y_absmax && !absmax_is_zero) {
    zero_word_kernel<<<1, 64, 0, st>>>(y_absmax);
    AQT_HIP(hipGetLastError());
  }
  const bool aligned = (reinterpret_cast<uintptr_t>(xq) % 16 == 0) && ws &&
                       (reinterpret_cast<uintptr_t>(ws) % 16 == 0) &&
                       (ws_is_prepared || reinterpret_cast<uintptr_t>(wq_packed) % 16 == 0);
  if (aligned && fwd_q_takes_fragments(M, K, N, epilogue)) {
    const int64_t nn = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
    const int64_t unit_wide = (epilogue == AQT_EPI_GLU) ? 128 : 256;
    v4i *wfrag = static_cast<v4i *>(ws);
    if (!ws_is_prepared) AQT_TRY(launch_prepare_weights(wq_packed, K, N, bits_w, ws, st));
    // 128 x 256 tiles need several rounds of them on the 512 workgroup slots to pay off (measured:
    // from about 2000 tiles at a fan-in of 512, from about 400 when the main loop is long), else 128 x 128
    const int64_t wide_tiles = cdiv(M, 128) * (N / 256);
    const bool wide = (nn % unit_wide == 0) && wide_tiles >= (K >= 1024 ? 384 : 2048);
    if (wide) {
      return packed ? launch_mfma_epi<2, 4, true>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st)
                    : launch_mfma_epi<2, 4, false>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st);
    }
    return packed ? launch_mfma_epi<2, 2, true>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st)
                  : launch_mfma_epi<2, 2, false>(epilogue, xq, s_x, wfrag, s_w, M, K, N, bias, y, acc_out, y_absmax, dact, st);
  }
  if (ws_is_prepared) return AQT_ERR_UNSUPPORTED;   // the general kernel reads the canonical operand
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  dense_fwd_general_kernel<<<static_cast<int>(cdiv(M * ncols, kThreads)), kThreads, 0, st>>>(
      xq, s_x, static_cast<const uint8_t *>(wq_packed), s_w, M, K, N, packed ? 1 : 0, bias, epilogue, y,
      acc_out, y_absmax, dact);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
