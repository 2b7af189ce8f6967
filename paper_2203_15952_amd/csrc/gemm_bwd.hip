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
//
// The weight-only forward (Sec. 4.1, configurations I8W / I4W: float32
// activations, integer weights) is the same kind of contraction and runs on the
// dX tile program:  y = act((x . wq) * s_w + bias).
#include <type_traits>

#include "aqt_internal.h"
#include "epilogue.h"

#ifdef AQT_TIMELINE
static __device__ long long g_timeline_bwd[AQT_TL_SLOTS * 8];
extern "C" int aqt_timeline_bwd(void *dst, size_t bytes) {
  return static_cast<int>(hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_timeline_bwd), bytes));
}
#endif

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

// int8 codes [K,N] -> bf16 (exact) in MFMA-fragment order, the dX kernel's second
// operand.  Fragment (jb, ks) covers fan-in rows 32*jb .. +31 and channels
// 16*ks .. +15; inside it lane (lk*32 + lr) owns the 8 consecutive channels
// 16*ks + 8*lk .. +7 of row 32*jb + lr, i.e. exactly what that lane feeds to
// v_mfma_f32_32x32x16_bf16.  A fragment is 1 KB, fragments are ordered
// [jb][ks], so a wavefront fetches one with a single fully coalesced 16-byte-per-lane load.
// With `packed` the input rows hold two int4 codes per byte (low nibble first), the
// layout of the forward weight operand for bits_w <= 4.
__global__ __launch_bounds__(kThreads) void codes_to_bf16_frag_kernel(const int8_t *__restrict__ codes, int K,
                                                                      int N, int packed, v4i *__restrict__ out) {
  const int64_t pieces = static_cast<int64_t>(K) * (N / 8);   // one 16-byte piece per (row, 8 channels)
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  const int ksteps = N / 16;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < pieces; i += stride) {
    // i enumerates the output in order: ((jb * ksteps + ks) * 64 + lane)
    const int lane = static_cast<int>(i & 63);
    const int64_t frag = i >> 6;
    const int ks = static_cast<int>(frag % ksteps), jb = static_cast<int>(frag / ksteps);
    const int k = 32 * jb + (lane & 31), n = 16 * ks + 8 * (lane >> 5);
    float f[8];
    if (packed) {
      const uint32_t w = *reinterpret_cast<const uint32_t *>(codes + static_cast<int64_t>(k) * (N >> 1) + (n >> 1));
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = static_cast<float>(static_cast<int>(w << (28 - 4 * e)) >> 28);
    } else {
      const v2i c = *reinterpret_cast<const v2i *>(codes + static_cast<int64_t>(k) * N + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        f[e] = static_cast<float>(static_cast<int8_t>(static_cast<uint32_t>(c.x) >> (8 * e)));
        f[4 + e] = static_cast<float>(static_cast<int8_t>(static_cast<uint32_t>(c.y) >> (8 * e)));
      }
    }
    v4i o;
    o.x = pack_bf16(f[0], f[1]); o.y = pack_bf16(f[2], f[3]);
    o.z = pack_bf16(f[4], f[5]); o.w = pack_bf16(f[6], f[7]);
    out[i] = o;
  }
}

// =====================================================================================
// dX = (dy * s_w) . wq^T       rows m, columns k, contraction over n
// Workgroup = 2 x WN wavefronts (WN = 2: two workgroups per CU; WN = 4: one), tile
// (64*TM) x (32*TN*WN), 32 n per stage.  The split operand sits on the short side
// of the wavefront tile (TM < TN).
//
// Data movement, chosen around what bounds this kernel on gfx950: LDS bandwidth
// (about 64 bytes per clock and CU for 16-byte reads), not the matrix cores.
//   * The bf16 codes never touch LDS.  They are stored in MFMA-fragment order
//     (codes_to_bf16_frag_kernel), so each wavefront pulls its 1 KB fragments
//     straight from L2 into registers with fully coalesced loads, one stage ahead.
//   * dy has to be scaled and split, so it is staged: global -> registers (two
//     alternating sets, a full stage in flight) -> bf16 hi/lo images in LDS (two
//     slots) -> MFMA fragments.  Its fragments live in one register set that is
//     refilled in place, each piece as soon as its last MFMA has issued.
//
// Software pipeline of one stage (per wavefront): two MFMA groups of 2*TM*TN, one
// per 16-deep fragment step.  Every other kind of work is cut into small pieces
// slotted between MFMA pairs, so that the LDS, vector-memory and VALU traffic of
// the next steps runs under the current MFMAs:
//   first half : MFMA(step 0) | refill dy fragments for step 1 | stage dy of the
//                next stage into the other LDS slot | fetch the codes of the next
//                stage, step 0
//   barrier    : the next stage's dy images are complete
//   second half: MFMA(step 1) | refill dy fragments for the next stage, step 0 |
//                fetch the codes of the next stage, step 1
// Loads past the last stage are clamped to it (harmless re-reads), so the loop
// body is branch-free and the interleaving below is what the hardware issues.
// LDS rows are 64 bytes without padding; their four 16-byte chunks are XOR-swizzled
// with bits 1..2 of the row so that 8 consecutive rows hit 8 different bank groups.
// =====================================================================================
constexpr int kSN = 32;      // contraction elements per stage
constexpr int kRowB = 64;    // LDS row: 32 bf16

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 3; }

#define AQT_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// s_waitcnt immediate (gfx9 layout): at most `vm` vector-memory and `lgkm` LDS
// operations of this wavefront may still be outstanding afterwards.
constexpr int waitcnt_imm(int vm, int lgkm) {
  return (vm & 0xF) | ((vm >> 4) << 14) | (7 << 4) | ((lgkm & 0xF) << 8);
}

// The same tile program serves the weight-only forward (integer weights, float32
// activations): there the float operand is x, the contraction runs over the fan-in,
// the codes are the forward weight operand, nothing is scaled on the way in, and the
// epilogue applies the per-channel scale, the bias and the activation.
//   MODE 0 / 1 : dX without / with a clip mask
//   MODE 2 + e : weight-only forward with epilogue e (none, Swish, GLU)
//   MODE 5     : dX without a clip mask, times an elementwise factor [M,K] on the way out (`bias` points at it):
//                the gradient that reaches the previous layer through its activation, with no pass of its own
// Names follow dX: `dy` is the float operand [M,N], N the contraction length, K the
// number of output columns (for GLU: value and gate channels together).
template <int TM, int TN, int MODE, int WN = 2>
__device__ __forceinline__ void f32_codes_tile(
    const float *__restrict__ dy, const v4i *__restrict__ wq_frag, const float *__restrict__ s_w,
    const float *__restrict__ s_x, const uint32_t *__restrict__ mask_x, const float *__restrict__ bias, int M,
    int K, int N, float *__restrict__ dx, int tiles_m, int tiles_c) {
  constexpr bool MASKED = (MODE == 1);
  constexpr bool WONLY = (MODE >= 2 && MODE <= 4);
  constexpr bool TIMES = (MODE == 5);
  constexpr int EPI = WONLY ? MODE - 2 : AQT_EPI_NONE;
  // Workgroup = 2 x WN wavefronts.  With WN = 4 the float operand tile is staged (and
  // scaled, split) once for four column wavefronts instead of two, which halves the
  // loads and the conversion arithmetic per MFMA.
  constexpr int NTHR = 64 * 2 * WN;        // threads
  constexpr int RP = NTHR / 8;               // rows staged per pass (8 threads per 32-float row piece)
  constexpr int BM = 64 * TM, BC = 32 * TN * WN;
  constexpr int kABytes = 2 * BM * kRowB;  // dy hi image, then dy lo image
  constexpr int NA = BM / RP;              // float4 of dy per thread per stage
  constexpr int P = TM * TN;               // MFMA pairs per half stage
  __shared__ __attribute__((aligned(1024))) uint8_t sA0[kABytes], sA1[kABytes];

  int id = blockIdx.x;
  const int total = tiles_m * tiles_c;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);  // one run of tiles per XCD
  const int bm = id / tiles_c, bc = id - bm * tiles_c;
  // A ragged last row tile is shifted up to end at row M: it recomputes a few rows
  // of its neighbour (same values, same addresses) instead of clamping loads.
  const int m0 = min(bm * BM, M - BM), c0 = bc * BC;

  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int lr = lane & 31, lk = lane >> 5;

  float4 ra[2][NA];
  float4 rs = {1.0f, 1.0f, 1.0f, 1.0f};

  // dy: a tile-uniform base (moves with the stage) plus small per-thread byte
  // offsets that stay fixed, so the loads can use scalar-base addressing.
  const char *a_base = reinterpret_cast<const char *>(dy + static_cast<int64_t>(m0) * N);
  const char *s_base = reinterpret_cast<const char *>(s_w);
  const uint32_t ga0 = static_cast<uint32_t>((t >> 3) * N + (t & 7) * 4) * 4u;  // piece i: + i * RP rows
  const uint32_t ga_step = static_cast<uint32_t>(RP * N) * 4u;
  const uint32_t gs = (t & 7) * 16u;
  // LDS offsets: piece i of a thread sits 32 rows below piece 0, which leaves the
  // swizzle bits of the row unchanged.
  const int ra0 = t >> 3, qa = t & 7;
  const int offa0 = ra0 * kRowB + (((qa >> 1) ^ swz(ra0)) << 4) + (qa & 1) * 8;

  // codes: fragment (jb, ks) starts at ((jb * N/16) + ks) * 64 pieces of 16 bytes;
  // this wavefront's column j-block is jb0 + j, a stage covers ks = 2*stage, 2*stage + 1.
  const int ksteps = N / 16;
  const int b_jstep = ksteps * 64;
  // First output channel of this wavefront's column block j.  A GLU tile pairs value
  // and gate channel blocks (even j: value, odd j: gate) so both meet in one lane.
  auto chan_of = [&](int j) -> int {
    const int cb = wn * TN + j;
    if (EPI == AQT_EPI_GLU) return ((cb & 1) ? (K >> 1) : 0) + bc * (BC / 2) + (cb >> 1) * 32;
    return c0 + cb * 32;
  };
  const v4i *b_lane = wq_frag + (static_cast<int64_t>(chan_of(0) / 32) * ksteps) * 64 + lane;
  // block j relative to block 0, in units of one block's fragments
  auto b_rel = [&](int j) -> int { return (EPI == AQT_EPI_GLU) ? (j & 1) * (K >> 6) + (j >> 1) : j; };

  auto load_s = [&](int n0) {
    if (!WONLY) rs = *reinterpret_cast<const float4 *>(s_base + n0 * 4 + gs);
  };
  auto load_a = [&](int set, int n0) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      ra[set][i] = *reinterpret_cast<const float4 *>(a_base + n0 * 4 + ga0 + i * ga_step);
  };
  auto store_a = [&](int set, int i, uint8_t *slot) {
    v2i hi, lo;
    uint32_t h, l;
    if (WONLY) {
      split_bf16(ra[set][i].x, ra[set][i].y, h, l); hi.x = h; lo.x = l;
      split_bf16(ra[set][i].z, ra[set][i].w, h, l); hi.y = h; lo.y = l;
    } else {
      split_bf16(ra[set][i].x * rs.x, ra[set][i].y * rs.y, h, l); hi.x = h; lo.x = l;
      split_bf16(ra[set][i].z * rs.z, ra[set][i].w * rs.w, h, l); hi.y = h; lo.y = l;
    }
    *reinterpret_cast<v2i *>(slot + offa0 + i * RP * kRowB) = hi;
    *reinterpret_cast<v2i *>(slot + BM * kRowB + offa0 + i * RP * kRowB) = lo;
  };

  v16f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // dy fragments: this lane's addresses.  Tile rows are multiples of 32 apart, so
  // the swizzle term depends on the lane only.
  const int sw = swz(lr);
  const int offk[2] = {((0 + lk) ^ sw) << 4, ((2 + lk) ^ sw) << 4};
  const int a_row = (wm * 32 * TM + lr) * kRowB;
  v4i fa[2 * TM];   // ah[0..TM-1], al[0..TM-1] of the fragment step in flight
  auto read_a = [&](const uint8_t *sA, int kk, int idx) {
    const int i = idx % TM, img = idx / TM;
    fa[idx] = *reinterpret_cast<const v4i *>(sA + img * BM * kRowB + a_row + i * 32 * kRowB + offk[kk]);
  };
  // codes fragments: one register set per (stage parity, fragment step)
  v4i fb[2][2][TN];
  auto load_b = [&](int par, int kk, int j, int stage) {
    fb[par][kk][j] = b_lane[static_cast<int64_t>(b_rel(j)) * b_jstep + (2 * stage + kk) * 64];
  };
  // MFMA number q of a half stage, q in [0, 2*P): all hi products first, then all
  // lo products, so that consecutive MFMAs never share an accumulator and each dy
  // fragment is used by TN consecutive MFMAs.
  auto mfma_q = [&](int par, int kk, int q) {
    const int tile = q % P, i = tile / TN, j = tile % TN;
    acc[i][j] = mfma_bf16(fa[(q < P ? 0 : TM) + i], fb[par][kk][j], acc[i][j]);
  };

  const int NT = N / kSN;
  auto stage_idx = [&](int s) { return s < NT - 1 ? s : NT - 1; };
  auto stage_n0 = [&](int s) { return stage_idx(s) * kSN; };

  AQT_TL_DECL;
  AQT_TL(0);
  // ---- prologue: stage 0 staged into slot 0, dy of stage 1 into register set 1,
  //      codes of stage 0 into their register sets ----
  load_s(0);
  load_a(0, 0);
#pragma unroll
  for (int j = 0; j < TN; ++j) { load_b(0, 0, j, 0); load_b(0, 1, j, 0); }
#pragma unroll
  for (int i = 0; i < NA; ++i) store_a(0, i, sA0);
  load_s(stage_n0(1));
  load_a(1, stage_n0(1));
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int idx = 0; idx < 2 * TM; ++idx) read_a(sA0, 0, idx);

  // One stage.  PAR = nt % 2 is a compile-time constant so that register sets
  // (stage s lives in set s % 2) are addressed statically.
  auto stage = [&](auto par, int nt) {
    constexpr int PAR = decltype(par)::value;
    uint8_t *curA = PAR ? sA1 : sA0;
    uint8_t *nxtA = PAR ? sA0 : sA1;
    const int s1 = stage_idx(nt + 1);
    // ---- first half: fragment step 0 ----
    // dy set PAR (emptied one stage ago) is refilled with stage nt + 2 while set PAR^1
    // (stage nt + 1, a full stage in flight by now) is staged below.
    load_a(PAR, stage_n0(nt + 2));
    AQT_SCHED_FENCE();
#pragma unroll
    for (int p = 0; p < P; ++p) {
      mfma_q(PAR, 0, 2 * p);
      mfma_q(PAR, 0, 2 * p + 1);
      AQT_SCHED_FENCE();
      // dy fragment idx is free once MFMA TN*(idx+1) - 1 has issued: refill it for step 1
#pragma unroll
      for (int idx = 0; idx < 2 * TM; ++idx)
        if (2 * p + 1 == TN * (idx + 1) - 1) read_a(curA, 1, idx);
#pragma unroll
      for (int c = (p * NA) / P; c < ((p + 1) * NA) / P; ++c) store_a(PAR ^ 1, c, nxtA);  // stage nt + 1
      if (p < TN) load_b(PAR ^ 1, 0, p, s1);
      AQT_SCHED_FENCE();
    }
    load_s(stage_n0(nt + 2));   // scales for the staging done one stage from now
    AQT_SCHED_FENCE();
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));   // own LDS traffic drained
    __builtin_amdgcn_s_barrier();
    // ---- second half: fragment step 1 ----
#pragma unroll
    for (int p = 0; p < P; ++p) {
      mfma_q(PAR, 1, 2 * p);
      mfma_q(PAR, 1, 2 * p + 1);
      AQT_SCHED_FENCE();
#pragma unroll
      for (int idx = 0; idx < 2 * TM; ++idx)
        if (2 * p + 1 == TN * (idx + 1) - 1) read_a(nxtA, 0, idx);   // stage nt + 1, step 0
      if (p < TN) load_b(PAR ^ 1, 1, p, s1);
      AQT_SCHED_FENCE();
    }
  };

  AQT_TL(1);
  int nt = 0;
  for (; nt + 1 < NT; nt += 2) {
    stage(std::integral_constant<int, 0>{}, nt);
    stage(std::integral_constant<int, 1>{}, nt + 1);
  }
  if (nt < NT) stage(std::integral_constant<int, 0>{}, nt);

  AQT_TL(2);
  // ---- epilogue: registers -> HBM.  Lane holds column (lane % 32) of each 32 x 32
  // tile, register r holds row 8*(r/4) + 4*(lane/32) + r%4; 32 lanes write 128
  // contiguous bytes.  Addresses are a uniform tile base plus one 32-bit lane offset;
  // the row and tile steps are compile-time multiples of K folded into the base.
  if (WONLY) {
    // de-quantize with the channel's scale, add the bias, apply the activation
    const int out_cols = (EPI == AQT_EPI_GLU) ? (K >> 1) : K;
    constexpr int JS = (EPI == AQT_EPI_GLU) ? 2 : 1;
    float *ybase = dx + static_cast<int64_t>(m0) * out_cols;
    const int row_l = wm * 32 * TM + 4 * lk;
#pragma unroll
    for (int j = 0; j < TN; j += JS) {
      const int n_a = chan_of(j) + lr;   // for GLU: the value channel = output column
      const float sc_a = s_w[n_a];
      const float bias_a = bias ? bias[n_a] : 0.0f;
      float sc_b = 0.0f, bias_b = 0.0f;
      if (EPI == AQT_EPI_GLU) {
        const int n_b = chan_of(j + 1) + lr;
        sc_b = s_w[n_b];
        bias_b = bias ? bias[n_b] : 0.0f;
      }
      const int lane_off = row_l * out_cols + n_a;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float v = acc[i][j][r] * sc_a + bias_a;
          float o;
          if (EPI == AQT_EPI_NONE) o = v;
          else if (EPI == AQT_EPI_SWISH) o = swish_f32(v);
          else o = v * sigmoid_f32(acc[i][j + (JS - 1)][r] * sc_b + bias_b);
          __builtin_nontemporal_store(o, ybase + (i * 32 + 8 * (r >> 2) + (r & 3)) * out_cols + lane_off);
        }
    }
    return;
  }
  float *obase = dx + static_cast<int64_t>(m0) * K + c0;
  const int lane_off = (wm * 32 * TM + 4 * lk) * K + wn * 32 * TN + lr;
  if (MASKED) {
    const int64_t tile0 = static_cast<int64_t>(m0) * K + c0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row_off = (i * 32 + 8 * (r >> 2) + (r & 3)) * K;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int off = row_off + j * 32 + lane_off;
          __builtin_nontemporal_store(mask_bit(mask_x, tile0 + off) ? acc[i][j][r] : 0.0f, obase + off);
        }
      }
  } else if (TIMES) {
    const float keep = (s_x[0] != 0.0f) ? 1.0f : 0.0f;
    const float *fbase = bias + static_cast<int64_t>(m0) * K + c0;   // the factor has dx's layout
    // the main loop's registers are free by now: all factors of a 32-row block are requested before the first is used
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float f[16][TN];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row_off = (i * 32 + 8 * (r >> 2) + (r & 3)) * K;
#pragma unroll
        for (int j = 0; j < TN; ++j) f[r][j] = __builtin_nontemporal_load(fbase + row_off + j * 32 + lane_off);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row_off = (i * 32 + 8 * (r >> 2) + (r & 3)) * K;
#pragma unroll
        for (int j = 0; j < TN; ++j)
          __builtin_nontemporal_store((keep != 0.0f) ? acc[i][j][r] * f[r][j] : 0.0f,
                                      obase + row_off + j * 32 + lane_off);
      }
    }
  } else {
    const float keep = (s_x[0] != 0.0f) ? 1.0f : 0.0f;   // NULL mask: "the scale is non-zero"
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row_off = (i * 32 + 8 * (r >> 2) + (r & 3)) * K;
#pragma unroll
        for (int j = 0; j < TN; ++j)
          __builtin_nontemporal_store((keep != 0.0f) ? acc[i][j][r] : 0.0f, obase + row_off + j * 32 + lane_off);
      }
  }
#ifdef AQT_TIMELINE
  AQT_TL(3);
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // the stores have been acknowledged
  AQT_TL(4);
  AQT_TL_WRITE(g_timeline_bwd, bm * 65536 + bc);
#endif
}

template <int TM, int TN, bool MASKED, int WN = 2>
__global__ __launch_bounds__(128 * WN, WN == 2 ? 2 : 1) void bwd_dx_mfma_kernel(
    const float *__restrict__ dy, const v4i *__restrict__ wq_frag, const float *__restrict__ s_w,
    const float *__restrict__ s_x, const uint32_t *__restrict__ mask_x, int M, int K, int N,
    float *__restrict__ dx, int tiles_m, int tiles_c) {
  f32_codes_tile<TM, TN, MASKED ? 1 : 0, WN>(dy, wq_frag, s_w, s_x, mask_x, nullptr, M, K, N, dx, tiles_m, tiles_c);
}

// dX times an elementwise factor of its own shape (no clip mask).
template <int TM, int TN, int WN = 2>
__global__ __launch_bounds__(128 * WN, WN == 2 ? 2 : 1) void bwd_dx_times_mfma_kernel(
    const float *__restrict__ dy, const v4i *__restrict__ wq_frag, const float *__restrict__ s_w,
    const float *__restrict__ s_x, const float *__restrict__ factor, int M, int K, int N, float *__restrict__ dx,
    int tiles_m, int tiles_c) {
  f32_codes_tile<TM, TN, 5, WN>(dy, wq_frag, s_w, s_x, nullptr, factor, M, K, N, dx, tiles_m, tiles_c);
}

// Weight-only forward (Sec. 4.1, I8W / I4W): y = act((x . wq) * s_w + bias), x float32 [M,K],
// codes in fragment order over [N][K].
template <int TM, int TN, int EPI, int WN = 2>
__global__ __launch_bounds__(128 * WN, WN == 2 ? 2 : 1) void dense_fwd_wonly_mfma_kernel(
    const float *__restrict__ x, const v4i *__restrict__ wq_frag, const float *__restrict__ s_w,
    const float *__restrict__ bias, int M, int K, int N, float *__restrict__ y, int tiles_m, int tiles_c) {
  f32_codes_tile<TM, TN, 2 + EPI, WN>(x, wq_frag, s_w, nullptr, nullptr, bias, M, N, K, y, tiles_m, tiles_c);
}

// =====================================================================================
// dW = s_x * xq^T . dy         rows k, columns n, contraction over m
// Neither operand is contraction-contiguous in memory, so each thread gathers a
// small block (4 k x 8 m of codes, 4 n x 4 m of gradients) with coalesced row-wise
// loads, transposes it in registers and writes m-contiguous pieces into LDS.
// The tile-local row index of the LDS images is de-interleaved, column 4*g + b
// lives in row b*(B/4) + g, so that the lanes of a wavefront write consecutive
// rows.  The contraction is split over row slabs of M; each workgroup writes a
// float32 partial tile and a second kernel folds the slabs in a fixed order
// (run-to-run reproducible), applies s_x and the mask.  The split operand (dy)
// sits on the short side of the wavefront tile (TC <= TR).
//
// Pipeline: as in the dX kernel.  Two LDS slots, one barrier per 32-row stage,
// two register sets so that every global load has a full stage in flight, and
// every other kind of work cut into pieces slotted between MFMA pairs:
//   first half : MFMA(step 0) | refill the code fragments in place for step 1,
//                fetch the dy fragments for step 1 | convert and stage the next
//                stage into the other LDS slot
//   barrier
//   second half: MFMA(step 1) | fragments of the next stage, step 0
// Rows past M (only in the last slab) are read from row M-1 and their codes are
// zeroed, so the loop body stays branch-free.
// =====================================================================================
// Workgroup = 2 x WNW wavefronts (WNW = 2: 256 x 128 tile, two workgroups per compute unit;
// WNW = 4: 256 x 256 tile, one workgroup of eight wavefronts per compute unit).  Two
// independent workgroups on a compute unit do not stay level: the older one is served first
// and the younger finishes its slab alone at about half the matrix pipe's rate (measured: 318 k
// against 407 k cycles for the two slabs of a pair).  Eight wavefronts behind one barrier
// cannot drift apart, so the wide form is used whenever the channel count allows it.
template <int TR, int TC, bool RAGGED, int WNW>  // tile is (64*TR) k-rows x (32*TC*WNW) n-columns; 32 m per stage
__global__ __launch_bounds__(128 * WNW, WNW == 2 ? 2 : 1) void bwd_dw_mfma_kernel(
    const int8_t *__restrict__ xq, const float *__restrict__ dy, int M, int K, int N, int m_per_slab,
    float *__restrict__ partial, int tiles_r, int tiles_c) {
  constexpr int NT = 128 * WNW;               // threads
  constexpr int BR = 64 * TR, BC = 32 * TC * WNW;
  constexpr int SM = 32;
  constexpr int GA = BR / 4, GB = BC / 4;   // 4-column groups per tile edge
  constexpr int P = TR * TC;                // MFMA pairs per half stage (2*TR*TC MFMAs)
  constexpr int RC = SM / (NT / 64);        // rows of m of the codes one thread gathers: 8 or 4
  static_assert(BR == 256 && P == 8 && NT / GB == 8, "the gather pattern below is written for 256-row tiles");
  // Two slots, each a codes image and a dy hi/lo image pair; after the main loop the same
  // memory stages the output tile.
  constexpr int kCBytes = BR * kRowB, kDBytes = 2 * BC * kRowB;
  __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * (kCBytes + kDBytes)];
  uint8_t *const sC0 = smem, *const sC1 = smem + kCBytes;
  uint8_t *const sD0 = smem + 2 * kCBytes, *const sD1 = smem + 2 * kCBytes + kDBytes;
  static_assert(2 * (kCBytes + kDBytes) >= 64 * BC * 4, "the output staging image must fit");

  // Workgroup -> (slab, tile).  All tiles of a slab read the same rows of xq and dy,
  // so a slab should live on one XCD (one L2) at one time: consecutive workgroup ids
  // are spread round-robin over the 8 XCDs, hence the remap to one contiguous run
  // of (slab, tile) pairs per XCD.
  const int tiles = tiles_r * tiles_c;
  int id = blockIdx.x;
  const int total = gridDim.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int slab = id / tiles;
  const int tile = id - slab * tiles;
  const int br = tile % tiles_r, bc = tile / tiles_r;   // row tiles of one column tile are neighbours
  const int r0 = br * BR, c0 = bc * BC;
  const int m_begin = slab * m_per_slab;
  const int m_end = min(M, m_begin + m_per_slab);

  const int t = threadIdx.x;
  const int wave = t >> 6, lane = t & 63;
  const int wm = wave / WNW, wn = wave % WNW;
  const int lr = lane & 31, lk = lane >> 5;

  // gather units: codes (g = t % 64: 4 k, mg = t / 64: RC m); gradients (h = t % GB: 4 n, ms = t / GB: 4 m)
  const int g = t & 63, mg = t >> 6;
  const int h = t % GB, ms = t / GB;
  uint32_t rx[2][RC];
  float4 ry[2][4];

  // Slab-uniform bases plus 32-bit offsets (a slab spans at most m_per_slab rows).
  const char *x_slab = reinterpret_cast<const char *>(xq + static_cast<int64_t>(m_begin) * K + r0);
  const char *y_slab = reinterpret_cast<const char *>(dy + static_cast<int64_t>(m_begin) * N + c0);
  const int m_last = M - 1 - m_begin;      // last valid row, slab-relative
  // RAGGED (M not a multiple of 32): rows past M are read from row M-1 and their codes zeroed.
  const uint32_t gx0 = static_cast<uint32_t>(mg * RC * K + 4 * g);
  const uint32_t gy0 = static_cast<uint32_t>(ms * 4 * N + 4 * h) * 4u;
  auto load_global = [&](int set, int mrel0) {
#pragma unroll
    for (int i = 0; i < RC; ++i) {
      if (RAGGED) {
        const int mrel = mrel0 + mg * RC + i;
        const int mc = min(mrel, m_last);
        const uint32_t v = *reinterpret_cast<const uint32_t *>(x_slab + static_cast<uint32_t>(mc * K + 4 * g));
        rx[set][i] = mrel <= m_last ? v : 0u;
      } else {
        rx[set][i] = *reinterpret_cast<const uint32_t *>(x_slab + static_cast<uint32_t>((mrel0 + i) * K) + gx0);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (RAGGED) {
        const int mc = min(mrel0 + ms * 4 + i, m_last);
        ry[set][i] = *reinterpret_cast<const float4 *>(y_slab + static_cast<uint32_t>(mc * N + 4 * h) * 4u);
      } else {
        ry[set][i] = *reinterpret_cast<const float4 *>(y_slab + static_cast<uint32_t>((mrel0 + i) * N) * 4u + gy0);
      }
    }
  };
  // LDS write offsets (row rho = b*G + g, swizzled 16-byte chunk); b adds whole multiples of
  // 32 rows, which leaves the swizzle bits unchanged.  A thread's piece of codes is RC bf16
  // along m: a whole chunk (RC = 8) or half of one (RC = 4).
  const int offc0 = g * kRowB + ((((mg * RC) >> 3) ^ swz(g)) << 4) + ((mg * RC) & 7) * 2;
  const int offd0 = h * kRowB + (((ms >> 1) ^ swz(h)) << 4) + (ms & 1) * 8;
  auto store_codes = [&](int set, int b, uint8_t *sC) {
    // byte b of the RC dwords -> RC bf16 along m
    float f[RC];
#pragma unroll
    for (int i = 0; i < RC; ++i) f[i] = static_cast<float>(static_cast<int8_t>(rx[set][i] >> (8 * b)));
    if (RC == 8) {
      v4i a;
      a.x = pack_bf16(f[0], f[1]); a.y = pack_bf16(f[2], f[3]);
      a.z = pack_bf16(f[4 % RC], f[5 % RC]); a.w = pack_bf16(f[6 % RC], f[7 % RC]);
      *reinterpret_cast<v4i *>(sC + offc0 + b * GA * kRowB) = a;
    } else {
      v2i a;
      a.x = pack_bf16(f[0], f[1]); a.y = pack_bf16(f[2], f[3]);
      *reinterpret_cast<v2i *>(sC + offc0 + b * GA * kRowB) = a;
    }
  };
  auto store_dy = [&](int set, int b, uint8_t *sD) {
    // component b of the four float4 -> hi/lo bf16 along m
    float y[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      y[i] = b == 0 ? ry[set][i].x : (b == 1 ? ry[set][i].y : (b == 2 ? ry[set][i].z : ry[set][i].w));
    v2i hi, lo;
    uint32_t hh, ll;
    split_bf16(y[0], y[1], hh, ll); hi.x = hh; lo.x = ll;
    split_bf16(y[2], y[3], hh, ll); hi.y = hh; lo.y = ll;
    *reinterpret_cast<v2i *>(sD + offd0 + b * GB * kRowB) = hi;
    *reinterpret_cast<v2i *>(sD + BC * kRowB + offd0 + b * GB * kRowB) = lo;
  };

  v16f acc[TR][TC];
#pragma unroll
  for (int i = 0; i < TR; ++i)
#pragma unroll
    for (int j = 0; j < TC; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragments: this lane's addresses (tile rows are multiples of 32 apart)
  const int sw = swz(lr);
  const int offk[2] = {((0 + lk) ^ sw) << 4, ((2 + lk) ^ sw) << 4};
  const int a_row = (wm * 32 * TR + lr) * kRowB;
  const int b_row = (wn * 32 * TC + lr) * kRowB;
  v4i fa[TR];            // code fragments of the step in flight, refilled in place
  v4i fb[2][2 * TC];     // dy fragments: [set][hi j..., lo j...]
  auto read_a = [&](const uint8_t *sC, int kk, int i) {
    fa[i] = *reinterpret_cast<const v4i *>(sC + a_row + i * 32 * kRowB + offk[kk]);
  };
  auto read_b = [&](const uint8_t *sD, int kk, int set, int idx) {
    const int j = idx % TC, img = idx / TC;
    fb[set][idx] = *reinterpret_cast<const v4i *>(sD + img * BC * kRowB + b_row + j * 32 * kRowB + offk[kk]);
  };
  // MFMA number q of a half stage, q in [0, 4*TR*TC/2... ): row tile i uses its code
  // fragment in 2*TC consecutive MFMAs (hi j0.., lo j0..), so it can be refilled right after.
  auto mfma_q = [&](int set, int q) {
    const int i = q / (2 * TC), w = q % (2 * TC), j = w % TC;
    acc[i][j] = mfma_bf16(fa[i], fb[set][w], acc[i][j]);
  };

  const int stages = (m_end - m_begin + SM - 1) / SM;
  auto stage_m = [&](int s) { return (s < stages - 1 ? s : stages - 1) * SM; };   // slab-relative

  AQT_TL_DECL;
  AQT_TL(0);
  // ---- prologue ----
  load_global(0, stage_m(0));
#pragma unroll
  for (int b = 0; b < 4; ++b) { store_codes(0, b, sC0); store_dy(0, b, sD0); }
  load_global(1, stage_m(1));
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int i = 0; i < TR; ++i) read_a(sC0, 0, i);
#pragma unroll
  for (int idx = 0; idx < 2 * TC; ++idx) read_b(sD0, 0, 0, idx);

  // One stage; PAR = s % 2 is a compile-time constant (register sets, LDS slots).
  // dy fragment sets alternate per half stage: step 0 uses fb[0], step 1 uses fb[1].
  auto stage = [&](auto par, int s) {
    constexpr int PAR = decltype(par)::value;
    uint8_t *curC = PAR ? sC1 : sC0, *curD = PAR ? sD1 : sD0;
    uint8_t *nxtC = PAR ? sC0 : sC1, *nxtD = PAR ? sD0 : sD1;
    // ---- first half: step 0 ----
    load_global(PAR, stage_m(s + 2));   // set PAR was consumed one stage ago
    AQT_SCHED_FENCE();
#pragma unroll
    for (int p = 0; p < P; ++p) {
      mfma_q(0, 2 * p);
      mfma_q(0, 2 * p + 1);
      AQT_SCHED_FENCE();
      if (p < 2 * TC) read_b(curD, 1, 1, p);                       // dy fragments for step 1
      if ((2 * p + 2) % (2 * TC) == 0) read_a(curC, 1, (2 * p + 1) / (2 * TC));   // row tile done: refill
      // stage s + 1 (register set PAR^1) into the other slot: 4 code pieces, 4 dy pieces
      if (p < 4) store_codes(PAR ^ 1, p, nxtC);
      else store_dy(PAR ^ 1, p - 4, nxtD);
      AQT_SCHED_FENCE();
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));   // own LDS traffic drained
    __builtin_amdgcn_s_barrier();
    // ---- second half: step 1 ----
#pragma unroll
    for (int p = 0; p < P; ++p) {
      mfma_q(1, 2 * p);
      mfma_q(1, 2 * p + 1);
      AQT_SCHED_FENCE();
      if (p < 2 * TC) read_b(nxtD, 0, 0, p);                       // next stage, step 0
      if ((2 * p + 2) % (2 * TC) == 0) read_a(nxtC, 0, (2 * p + 1) / (2 * TC));
      AQT_SCHED_FENCE();
    }
  };

  AQT_TL(1);
  int s = 0;
  for (; s + 1 < stages; s += 2) {
    stage(std::integral_constant<int, 0>{}, s);
    stage(std::integral_constant<int, 1>{}, s + 1);
  }
  if (s < stages) stage(std::integral_constant<int, 0>{}, s);
  AQT_TL(2);

  // ---- epilogue: partial tile -> workspace.
  // Written lane by lane the tile would reach HBM as 4-byte pieces at a 16-byte stride (the
  // de-interleaved columns), which the memory system turns into several times the traffic,
  // all of it in the tail of the launch.  So the tile goes through LDS (free by now) and
  // leaves as whole rows.  Accumulator row rho = wm*128 + i*32 + local (local = 8*(r/4) +
  // r%4 + 4*lk) is tile row 4*(rho % 64) + rho / 64 and accumulator column rho_c =
  // wn*32*TC + j*32 + lr is tile column 4*(rho_c % GB) + rho_c / GB (the de-interleaving of
  // the staging).  Pass p (0..3) moves the 64 tile rows 4*q + p: they belong to the
  // wavefronts with wm = p / 2 and their row blocks i = 2*(p % 2), 2*(p % 2) + 1, q = (i % 2)*32 + local.
  float *out = partial + static_cast<int64_t>(slab) * K * N + static_cast<int64_t>(r0) * N + c0;
  float *img = reinterpret_cast<float *>(smem);   // [64][BC]
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    __syncthreads();   // operand fragments (p = 0) or the previous pass's rows have been read by everybody
    if (wm == (p >> 1)) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        const int i = 2 * (p & 1) + ii;
#pragma unroll
        for (int j = 0; j < TC; ++j) {
          const int rho_c = wn * 32 * TC + j * 32 + lr;
          const int n_l = 4 * (rho_c % GB) + rho_c / GB;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int q = ii * 32 + 8 * (r >> 2) + (r & 3) + 4 * lk;
            img[q * BC + n_l] = acc[i][j][r];
          }
        }
      }
    }
    __syncthreads();
    // 64 rows x BC floats as float4: BC/4 threads per row
#pragma unroll
    for (int it = 0; it < 64 * (BC / 4) / NT; ++it) {
      const int idx = t + it * NT;
      const int q = idx / (BC / 4), c4 = idx % (BC / 4);
      const float4 v = *reinterpret_cast<const float4 *>(img + q * BC + c4 * 4);
      *reinterpret_cast<float4 *>(out + (4 * q + p) * N + c4 * 4) = v;
    }
  }
#ifdef AQT_TIMELINE
  AQT_TL(3);
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // the stores have been acknowledged
  AQT_TL(4);
  AQT_TL_WRITE(g_timeline_bwd, slab * 65536 + tile);
#endif
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
  bool dx_wide;    // 128 x 256 tiles (else 128 x 128)
  bool dx_wide8;   // 128 x 512 tiles, eight wavefronts: the gradient tile is staged once for four column wavefronts
  bool dw_wide8;   // dW on 256 x 256 tiles, eight wavefronts
  int slabs;
  int m_per_slab;
  size_t off_bf, off_part, off_bias, total;
};

BwdPlan plan_bwd(int64_t M, int64_t K, int64_t N) {
  BwdPlan p{};
  const bool fits32 = M < (int64_t(1) << 31) / (K > N ? K : N);
  // dX: columns are K, contraction N in stages of 32; row tiles of 128 (the last one may be shifted)
  p.dx_mfma = fits32 && (N % kSN == 0) && (K % 128 == 0) && (M >= 128);
  p.dx_wide = (K % 256 == 0) && cdiv(M, 128) * (K / 256) >= 512;
  p.dx_wide8 = p.dx_wide && (K % 512 == 0) && cdiv(M, 128) * (K / 512) >= 256;
  // dW: 256 x 256 tiles (eight wavefronts, one workgroup per compute unit) when N allows, else 256 x 128
  // (two per compute unit); slabs over M so that the launch fills the chip once
  p.dw_mfma = fits32 && (K % 256 == 0) && (N % 128 == 0);
  p.dw_wide8 = p.dw_mfma && (N % 256 == 0);
  const int64_t tiles = p.dw_mfma ? (K / 256) * (N / (p.dw_wide8 ? 256 : 128)) : 1;
  int64_t slabs = p.dw_mfma ? cdiv(p.dw_wide8 ? 256 : 512, tiles) : 1;
  if (slabs > 64) slabs = 64;
  int64_t per = cdiv(M, slabs);
  per = cdiv(per, 32) * 32;            // whole stages
  slabs = cdiv(M, per);
  if (per * (K > N ? K : N) >= (int64_t(1) << 30)) p.dw_mfma = false;   // 32-bit byte offsets inside a slab
  p.slabs = static_cast<int>(slabs);
  p.m_per_slab = static_cast<int>(per);
  size_t off = 0;
  p.off_bf = off;   off += align_up(static_cast<size_t>(K) * N * 2, 256);
  p.off_part = off; off += align_up(static_cast<size_t>(p.slabs) * K * N * 4, 256);
  p.off_bias = off; off += align_up(static_cast<size_t>(kBiasSlabs) * N * sizeof(double), 256);
  p.total = off;
  return p;
}

template <int TM, int TN, int WN = 2>
aqt_status launch_dx(const float *dy, const v4i *wq_frag, const aqt_saved *sv, int64_t M, int64_t K, int64_t N,
                     float *dx, hipStream_t st, const float *factor = nullptr) {
  constexpr int BM = 64 * TM, BC = 32 * TN * WN;
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_c = static_cast<int>(K / BC);
  if (factor) {   // the caller has checked that there is no clip mask
    bwd_dx_times_mfma_kernel<TM, TN, WN><<<tiles_m * tiles_c, 128 * WN, 0, st>>>(
        dy, wq_frag, sv->s_w, sv->s_x, factor, static_cast<int>(M), static_cast<int>(K), static_cast<int>(N), dx,
        tiles_m, tiles_c);
    AQT_HIP(hipGetLastError());
    return AQT_OK;
  }
  auto kern = sv->mask_x ? bwd_dx_mfma_kernel<TM, TN, true, WN> : bwd_dx_mfma_kernel<TM, TN, false, WN>;
  kern<<<tiles_m * tiles_c, 128 * WN, 0, st>>>(dy, wq_frag, sv->s_w, sv->s_x, sv->mask_x, static_cast<int>(M),
                                                  static_cast<int>(K), static_cast<int>(N), dx, tiles_m, tiles_c);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

template <int TR, int TC, int WNW>
aqt_status launch_dw(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N, const BwdPlan &p,
                     float *partial, hipStream_t st) {
  constexpr int BR = 64 * TR, BC = 32 * TC * WNW;
  auto kern = (M % 32 == 0) ? bwd_dw_mfma_kernel<TR, TC, false, WNW> : bwd_dw_mfma_kernel<TR, TC, true, WNW>;
  const int tiles_r = static_cast<int>(K / BR), tiles_c = static_cast<int>(N / BC);
  kern<<<tiles_r * tiles_c * p.slabs, 128 * WNW, 0, st>>>(sv->xq, dy, static_cast<int>(M), static_cast<int>(K),
                                                         static_cast<int>(N), p.m_per_slab, partial, tiles_r,
                                                         tiles_c);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

// Weight-only forward for any shape: one thread per output, the de-quantized weight
// rounded to float32 as a float graph would hold it, products summed in float64.
__global__ __launch_bounds__(kThreads) void dense_fwd_wonly_general_kernel(
    const float *__restrict__ x, const uint8_t *__restrict__ wq, const float *__restrict__ s_w, int64_t M,
    int64_t K, int64_t N, int packed, const float *__restrict__ bias, int epilogue, float *__restrict__ y) {
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (idx >= M * ncols) return;
  const int64_t m = idx / ncols, j = idx - m * ncols;
  const int64_t row_bytes = packed ? (K + 1) / 2 : K;
  const int parts = (epilogue == AQT_EPI_GLU) ? 2 : 1;
  float v[2];
  for (int p = 0; p < parts; ++p) {
    const int64_t n = j + p * ncols;
    double s = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      int c;
      if (packed) {
        const uint32_t b = wq[n * row_bytes + (k >> 1)];
        c = static_cast<int>(((k & 1) ? (b >> 4) : (b & 0xFu)) << 28) >> 28;
      } else {
        c = static_cast<int8_t>(wq[n * row_bytes + k]);
      }
      s += static_cast<double>(x[m * K + k]) * static_cast<double>(s_w[n] * static_cast<float>(c));
    }
    float t = static_cast<float>(s);
    if (bias) t = t + bias[n];
    v[p] = t;
  }
  float out;
  if (epilogue == AQT_EPI_NONE) out = v[0];
  else if (epilogue == AQT_EPI_SWISH) out = swish_f32(v[0]);
  else out = v[0] * sigmoid_f32(v[1]);
  y[m * ncols + j] = out;
}

template <int TM, int TN, int WN = 2>
aqt_status launch_wonly(const float *x, const v4i *frag, const float *s_w, const float *bias, int epilogue,
                        int64_t M, int64_t K, int64_t N, float *y, hipStream_t st) {
  constexpr int BM = 64 * TM, BC = 32 * TN * WN;
  const int tiles_m = static_cast<int>(cdiv(M, BM)), tiles_c = static_cast<int>(N / BC);
  auto kern = (epilogue == AQT_EPI_NONE)    ? dense_fwd_wonly_mfma_kernel<TM, TN, AQT_EPI_NONE, WN>
              : (epilogue == AQT_EPI_SWISH) ? dense_fwd_wonly_mfma_kernel<TM, TN, AQT_EPI_SWISH, WN>
                                            : dense_fwd_wonly_mfma_kernel<TM, TN, AQT_EPI_GLU, WN>;
  kern<<<tiles_m * tiles_c, 128 * WN, 0, st>>>(x, frag, s_w, bias, static_cast<int>(M), static_cast<int>(K),
                                                  static_cast<int>(N), y, tiles_m, tiles_c);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace

size_t fwd_wonly_workspace_bytes(int64_t K, int64_t N) { return align_up(static_cast<size_t>(K) * N * 2, 256); }

aqt_status launch_dense_fwd_wonly(const float *x, const void *wq_packed, const float *s_w, int64_t M, int64_t K,
                                  int64_t N, int bits_w, const float *bias, int epilogue, float *y, void *ws,
                                  hipStream_t st) {
  const bool packed = packed4(bits_w);
  const bool fits32 = M < (int64_t(1) << 30) / (K > N ? K : N);
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(wq_packed) % 8 == 0 &&
                       ws && reinterpret_cast<uintptr_t>(ws) % 16 == 0;
  // column tiles of 128 channels (64 value + 64 gate channels for GLU), 256 when there are enough of them
  const int64_t nn = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  const int64_t unit = (epilogue == AQT_EPI_GLU) ? 64 : 128;
  if (fits32 && aligned && M >= 128 && K % kSN == 0 && nn % unit == 0) {
    v4i *frag = static_cast<v4i *>(ws);
    const int64_t pieces = N * (K / 8);
    int g = static_cast<int>(cdiv(pieces, kThreads));
    if (g > 2048) g = 2048;
    codes_to_bf16_frag_kernel<<<g, kThreads, 0, st>>>(static_cast<const int8_t *>(wq_packed), static_cast<int>(N),
                                                      static_cast<int>(K), packed ? 1 : 0, frag);
    AQT_HIP(hipGetLastError());
    const bool wide = (nn % (2 * unit) == 0) && cdiv(M, 128) * (N / 256) >= 512;
    const bool wide8 = wide && (nn % (4 * unit) == 0) && cdiv(M, 128) * (N / 512) >= 256;   // eight wavefronts
    if (wide8) return launch_wonly<2, 4, 4>(x, frag, s_w, bias, epilogue, M, K, N, y, st);
    if (wide) return launch_wonly<2, 4>(x, frag, s_w, bias, epilogue, M, K, N, y, st);
    return launch_wonly<2, 2>(x, frag, s_w, bias, epilogue, M, K, N, y, st);
  }
  const int64_t ncols = (epilogue == AQT_EPI_GLU) ? N / 2 : N;
  dense_fwd_wonly_general_kernel<<<static_cast<int>(cdiv(M * ncols, kThreads)), kThreads, 0, st>>>(
      x, static_cast<const uint8_t *>(wq_packed), s_w, M, K, N, packed ? 1 : 0, bias, epilogue, y);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

size_t bwd_workspace_bytes(int64_t M, int64_t K, int64_t N) { return plan_bwd(M, K, N).total; }

aqt_status launch_dense_bwd(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N, float *dx,
                            float *dw, float *dbias, void *ws, size_t ws_bytes, hipStream_t st,
                            const float *dx_factor) {
  (void)ws_bytes;
  const BwdPlan p = plan_bwd(M, K, N);
  uint8_t *base = static_cast<uint8_t *>(ws);
  // 16-byte vector accesses on dy and on the buffers carved from the workspace (their
  // offsets are multiples of 256); anything else takes the general kernels
  const bool dy_aligned = reinterpret_cast<uintptr_t>(dy) % 16 == 0 && reinterpret_cast<uintptr_t>(ws) % 16 == 0;
  if (dx) {
    if (p.dx_mfma && dy_aligned && reinterpret_cast<uintptr_t>(sv->s_w) % 16 == 0 &&
        reinterpret_cast<uintptr_t>(sv->wq_kn) % 8 == 0) {
      v4i *wq_frag = reinterpret_cast<v4i *>(base + p.off_bf);
      const int64_t pieces = K * (N / 8);
      int g = static_cast<int>(cdiv(pieces, kThreads));
      if (g > 2048) g = 2048;
      codes_to_bf16_frag_kernel<<<g, kThreads, 0, st>>>(sv->wq_kn, static_cast<int>(K), static_cast<int>(N), 0, wq_frag);
      AQT_HIP(hipGetLastError());
      // the factor rides in the epilogue when there is no clip mask and it can be read like dx is written
      const float *fused = (dx_factor && !sv->mask_x) ? dx_factor : nullptr;
      if (p.dx_wide8) AQT_TRY((launch_dx<2, 4, 4>(dy, wq_frag, sv, M, K, N, dx, st, fused)));
      else if (p.dx_wide) AQT_TRY((launch_dx<2, 4>(dy, wq_frag, sv, M, K, N, dx, st, fused)));
      else AQT_TRY((launch_dx<2, 2>(dy, wq_frag, sv, M, K, N, dx, st, fused)));
      if (dx_factor && !fused) AQT_TRY(launch_dact_mul(dx, dx_factor, M, K, K, dx, st));
    } else {
      bwd_dx_general_kernel<<<static_cast<int>(cdiv(M * K, kThreads)), kThreads, 0, st>>>(
          dy, sv->wq_kn, sv->s_w, sv->s_x, sv->mask_x, M, K, N, dx);
      AQT_HIP(hipGetLastError());
      if (dx_factor) AQT_TRY(launch_dact_mul(dx, dx_factor, M, K, K, dx, st));
    }
  }
  if (dw) {
    if (p.dw_mfma && dy_aligned && reinterpret_cast<uintptr_t>(sv->xq) % 4 == 0 &&
        reinterpret_cast<uintptr_t>(dw) % 16 == 0) {
      float *partial = reinterpret_cast<float *>(base + p.off_part);
      if (p.dw_wide8) AQT_TRY((launch_dw<4, 2, 4>(dy, sv, M, K, N, p, partial, st)));
      else AQT_TRY((launch_dw<4, 2, 2>(dy, sv, M, K, N, p, partial, st)));
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
