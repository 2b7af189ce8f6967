// The float core of the Conformer self-attention module between its two quantized
// projections (arxiv 2203.15952, Sec. 3.2: 4 or 8 heads; Sec. 3.3: a limited left context
// and, in the non-causal encoder, a limited right context): for every utterance, head and
// query frame, softmax over the key frames of the window of the scaled dot products, times
// the values.  Float32 throughout: both contractions run on the float32 matrix cores
// (v_mfma_f32_32x32x2_f32: exact products, float32 accumulation), with an online softmax
// (running maximum and sum per query, the output rescaled when the maximum moves), so the
// scores never leave the chip; the largest |result| is reduced on the way out for the
// quantizer of the output projection (Fig. 2).
//
// qkv [B*T, 3D]: queries, keys, values in three column blocks of width D, head h in columns
// h*dh .. (h+1)*dh of each.  A workgroup owns 128 query frames of one utterance and head, a
// wavefront 32 of them, and all walk the key frames of their windows 64 at a time.  Both
// products are formed transposed, so that a lane owns one query from start to end:
//   S^T (64 keys x 32 queries) = K Q_w^T   A operand: keys from LDS; B operand: the wavefront's
//                                          queries, held in 32 registers per lane for the whole kernel
//   a lane then holds 32 scores of ITS query: maximum, exponentials and sum are lane-local (one
//   exchange with the other half of the wavefront per step)
//   O^T (64 x 32 queries) += V^T P^T       B operand: the probabilities, exactly where the first
//                                          product left them; A operand: values from LDS
// so the probabilities never leave the registers and the running maximum, the rescaling of O
// and the final division need no cross-lane traffic.  An MFMA step contracts two positions,
// lane half lk supplying the second index lk: key and query rows are stored "parity-major"
// along the head (even positions, then odd ones) so that each lane finds its 32 values
// contiguous and fetches them 16 bytes at a time; in the second product the step (nb, r) pairs
// the keys 32 nb + 8 (r / 4) + r % 4 and that + 4, which is where the accumulator layout of
// the first product put them.  LDS rows are 68 floats: 16-byte aligned, and rows map to
// different banks.  The result leaves through LDS as whole rows.
#include "aqt_internal.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;
constexpr int kQ = 128;         // query frames per workgroup (32 per wavefront)
constexpr int kK = 64;          // key frames per step
constexpr int kDh = 64;         // widest head a tile holds; narrower heads are padded with zeros
constexpr int kLd = kDh + 4;    // LDS row stride in floats
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct AttnGeom {
  int64_t B, T, D;
  int heads, dh, left, right;   // left / right < 0: no limit on that side
  int qtiles;                   // 128-frame query tiles per utterance
  float scale_log2e;            // log2(e) / sqrt(dh): scores are kept in the exponent domain of exp2
  float scale;                  // 1 / sqrt(dh)
};

__device__ __forceinline__ int parity_major(int c) { return (c & 1) * 32 + (c >> 1); }

__device__ __forceinline__ uint32_t wave_max_bits(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), off, 64));
    v = v > o ? v : o;
  }
  return v;
}

// 64 frames x 64 head columns starting at frame row0 and column col0 of a [B*T, ld_src] matrix into dst[frame][col] (col in
// parity-major order if asked); frames beyond the utterance and columns beyond the head are zero.
// Loads go to clamped, always valid addresses (no branches, sixteen in flight per thread).
__device__ __forceinline__ void stage_tile(float *__restrict__ dst, const float *__restrict__ src, int64_t ld_src,
                                           const AttnGeom &g, int64_t b, int64_t row0, int64_t col0, bool permute) {
  const int d = threadIdx.x & 63, r0 = threadIdx.x >> 6;
  const int dd = d < g.dh ? d : g.dh - 1;
  const int at = permute ? parity_major(d) : d;
  float v[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    int64_t t = row0 + r0 + 4 * k;
    t = t < g.T ? t : g.T - 1;
    v[k] = src[(b * g.T + t) * ld_src + col0 + dd];
  }
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = r0 + 4 * k;
    dst[r * kLd + at] = (d < g.dh && row0 + r < g.T) ? v[k] : 0.0f;
  }
}

// The two halves of stage_tile, so that the loads of the next step can be in flight while this step is
// being computed: sixteen clamped loads into registers, and later the sixteen LDS writes (with the zeros).
__device__ __forceinline__ void load_tile(float (&v)[16], const float *__restrict__ src, int64_t ld_src,
                                          const AttnGeom &g, int64_t b, int64_t row0, int64_t col0) {
  const int d = threadIdx.x & 63, r0 = threadIdx.x >> 6;
  const int dd = d < g.dh ? d : g.dh - 1;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    int64_t t = row0 + r0 + 4 * k;
    t = t < g.T ? t : g.T - 1;
    v[k] = src[(b * g.T + t) * ld_src + col0 + dd];
  }
}
__device__ __forceinline__ void store_tile(float *__restrict__ dst, const float (&v)[16], const AttnGeom &g,
                                           int64_t row0, bool permute) {
  const int d = threadIdx.x & 63, r0 = threadIdx.x >> 6;
  const int at = permute ? parity_major(d) : d;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = r0 + 4 * k;
    dst[r * kLd + at] = (d < g.dh && row0 + r < g.T) ? v[k] : 0.0f;
  }
}

__global__ __launch_bounds__(kThreads, 2) void attention_fwd_kernel(const float *__restrict__ qkv, AttnGeom g,
                                                                 float *__restrict__ ctx,
                                                                 uint32_t *__restrict__ absmax,
                                                                 float *__restrict__ lse) {
  __shared__ __attribute__((aligned(16))) float lds[2 * kK * kLd];
  float *Ks = lds;              // keys, parity-major along the head
  float *Vs = lds + kK * kLd;   // values
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lk = lane >> 5;
  int64_t id = blockIdx.x;
  const int qt = static_cast<int>(id % g.qtiles);
  id /= g.qtiles;
  const int h = static_cast<int>(id % g.heads);
  const int64_t b = id / g.heads;
  const int64_t t0 = static_cast<int64_t>(qt) * kQ;
  const int64_t hc = static_cast<int64_t>(h) * g.dh;

  // the wavefront's 32 queries as a B operand: lane (lr, lk) keeps Q[query lr][2 i + lk], i < 32
  stage_tile(Ks, qkv, 3 * g.D, g, b, t0, hc, true);
  stage_tile(Vs, qkv, 3 * g.D, g, b, t0 + 64, hc, true);
  __syncthreads();
  float qf[32];
  {
    const float *src = (wave < 2 ? Ks : Vs) + ((wave & 1) * 32 + lr) * kLd + lk * 32;
#pragma unroll
    for (int i4 = 0; i4 < 8; ++i4) {
      const v4f q = *reinterpret_cast<const v4f *>(src + 4 * i4);
      qf[4 * i4] = q.x; qf[4 * i4 + 1] = q.y; qf[4 * i4 + 2] = q.z; qf[4 * i4 + 3] = q.w;
    }
  }
  const int64_t tw = t0 + wave * 32;          // first query frame of this wavefront
  const bool active = tw < g.T;               // idle wavefronts of a ragged tile still stage and meet the barriers
  const int64_t t = tw + lr;                  // this lane's query frame

  // key frames any query of this tile may look at
  const int64_t tlast = (t0 + kQ - 1 < g.T ? t0 + kQ - 1 : g.T - 1);
  const int64_t jmin = (g.left < 0 || t0 - g.left < 0) ? 0 : t0 - g.left;
  const int64_t jmax = (g.right < 0 || tlast + g.right > g.T - 1) ? g.T - 1 : tlast + g.right;
  const int64_t wlo = g.left < 0 ? 0 : t - g.left;                       // this query's window
  const int64_t whi = (g.right < 0 || t + g.right > g.T - 1) ? g.T - 1 : t + g.right;

  float m = -1e30f, l = 0.0f;   // running maximum (exponent domain of exp2); this lane's share of the running sum
  v16f o[2];                    // element r: head column 32 blk + 8 (r / 4) + 4 lk + r % 4 of this lane's query
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    o[0][r] = 0.0f;
    o[1][r] = 0.0f;
  }
  float kn[16], vn[16];   // keys and values of the next step, on their way from memory while this step computes
  const int64_t jfirst = jmin / kK * kK;
  load_tile(kn, qkv, 3 * g.D, g, b, jfirst, g.D + hc);
  load_tile(vn, qkv, 3 * g.D, g, b, jfirst, 2 * g.D + hc);
  for (int64_t j0 = jfirst; j0 <= jmax; j0 += kK) {
    __syncthreads();   // the queries have been taken / the previous step's reads of Ks and Vs are over
    store_tile(Ks, kn, g, j0, true);
    store_tile(Vs, vn, g, j0, false);
    __syncthreads();
    if (j0 + kK <= jmax) {
      load_tile(kn, qkv, 3 * g.D, g, b, j0 + kK, g.D + hc);
      load_tile(vn, qkv, 3 * g.D, g, b, j0 + kK, 2 * g.D + hc);
    }
    if (active) {
      // s[nb][r]: score of key j0 + 32 nb + 8 (r / 4) + 4 lk + r % 4 against this lane's query
      v16f s[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[nb][r] = 0.0f;
        const float *kp = Ks + (nb * 32 + lr) * kLd + lk * 32;
#pragma unroll
        for (int i4 = 0; i4 < 8; ++i4) {
          const v4f k = *reinterpret_cast<const v4f *>(kp + 4 * i4);
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(k.x, qf[4 * i4], s[nb], 0, 0, 0);
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(k.y, qf[4 * i4 + 1], s[nb], 0, 0, 0);
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(k.z, qf[4 * i4 + 2], s[nb], 0, 0, 0);
          s[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(k.w, qf[4 * i4 + 3], s[nb], 0, 0, 0);
        }
      }
      // window, running maximum, probabilities
      float mx = -1e30f;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t j = j0 + 32 * nb + 8 * (r >> 2) + 4 * lk + (r & 3);
          const float x = (j >= wlo && j <= whi) ? s[nb][r] * g.scale_log2e : -1e30f;
          s[nb][r] = x;
          mx = fmaxf(mx, x);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mnew = fmaxf(m, mx);
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      m = mnew;
      float sum = 0.0f;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = s[nb][r] > -1e29f ? __builtin_amdgcn_exp2f(s[nb][r] - mnew) : 0.0f;
          s[nb][r] = p;
          sum += p;
        }
      l = l * alpha + sum;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o[0][r] *= alpha;
        o[1][r] *= alpha;
      }
      // O^T += V^T P^T: step (nb, r) contracts the keys 32 nb + 8 (r / 4) + r % 4 (lk = 0) and that + 4 (lk = 1)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float *vp = Vs + (32 * nb + 8 * (r >> 2) + 4 * lk + (r & 3)) * kLd + lr;
          o[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(vp[0], s[nb][r], o[0], 0, 0, 0);
          o[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(vp[32], s[nb][r], o[1], 0, 0, 0);
        }
    }
  }
  // out through LDS, so that rows leave as whole 256-byte pieces
  __syncthreads();
  float *ot = lds + wave * 32 * kLd;   // [32 queries][68], this wavefront's own quarter
  uint32_t amax = 0u;
  if (active) {
    const float lt = l + __shfl_xor(l, 32, 64);
    const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
    // what the backward needs to form the probabilities again: p = exp2(score - lse)
    if (lse && lk == 0 && t < g.T) lse[(b * g.T + t) * g.heads + h] = m + log2f(lt);
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        v4f v;
        v.x = o[blk][4 * r4] * inv; v.y = o[blk][4 * r4 + 1] * inv;
        v.z = o[blk][4 * r4 + 2] * inv; v.w = o[blk][4 * r4 + 3] * inv;
        *reinterpret_cast<v4f *>(ot + lr * kLd + 32 * blk + 8 * r4 + 4 * lk) = v;
      }
    __builtin_amdgcn_wave_barrier();   // the wavefront's own LDS writes above, its own reads below
    for (int q = 0; q < 32; ++q) {
      if (tw + q < g.T && lane < g.dh) {
        const float v = ot[q * kLd + lane];
        ctx[(b * g.T + tw + q) * g.D + hc + lane] = v;
        amax = max(amax, __float_as_uint(v) & 0x7FFFFFFFu);
      }
    }
  }
  if (absmax) {   // uniform: the word only grows, so a stale read can only cost a redundant atomic
    amax = wave_max_bits(amax);
    if (lane == 0 && amax > *reinterpret_cast<volatile uint32_t *>(absmax)) atomicMax(absmax, amax);
  }
}

// ---- backward -------------------------------------------------------------------------------
// With P = softmax rows (formed again from the scores and the saved lse), dP = dO V^T and
// D_t = dO_t . O_t:   dS = P (dP - D);  dQ = dS K / sqrt(dh);  dK = dS^T Q / sqrt(dh);  dV = P^T dO.
// Two kernels in the forward's style, each with a lane owning the row it accumulates, so no sum is
// shared between workgroups and every result has one fixed summation order:
//   dq kernel: a lane owns a query.  S^T = K Q^T and dP^T = V dO^T leave its scores and dP in
//     registers, dS is lane-local, dQ^T += K^T dS^T takes dS as B operand where it stands.
//   dk/dv kernel: a lane owns a key.  S = Q K^T and dP = dO V^T (keys and values of the tile held in
//     registers as B operands), then dV^T += dO^T P and dK^T += Q^T dS.

// D[b,t,h] = sum_d dctx[b,t,h dh + d] * ctx[b,t,h dh + d]; one wavefront per token
__global__ __launch_bounds__(kThreads) void attention_rowdot_kernel(const float *__restrict__ dctx,
                                                                    const float *__restrict__ ctx, AttnGeom g,
                                                                    float *__restrict__ dsum) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t M = g.B * g.T;
  for (int64_t m = static_cast<int64_t>(blockIdx.x) * 4 + wave; m < M; m += static_cast<int64_t>(gridDim.x) * 4)
    for (int h = 0; h < g.heads; ++h) {
      const int64_t at = m * g.D + static_cast<int64_t>(h) * g.dh + lane;
      float v = lane < g.dh ? dctx[at] * ctx[at] : 0.0f;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0) dsum[m * g.heads + h] = v;
    }
}

// the 32 rows of a wavefront out of a staged tile pair as a B operand: lane (lr, lk) gets row lr, positions 2 i + lk
__device__ __forceinline__ void take_rows(float (&f)[32], const float *lo, const float *hi, int wave, int lr, int lk) {
  const float *src = (wave < 2 ? lo : hi) + ((wave & 1) * 32 + lr) * kLd + lk * 32;
#pragma unroll
  for (int i4 = 0; i4 < 8; ++i4) {
    const v4f q = *reinterpret_cast<const v4f *>(src + 4 * i4);
    f[4 * i4] = q.x; f[4 * i4 + 1] = q.y; f[4 * i4 + 2] = q.z; f[4 * i4 + 3] = q.w;
  }
}

// acc (64 x 32, two blocks) = A B with A: 32-row blocks of an LDS tile (parity-major rows), B: 32 registers per lane
__device__ __forceinline__ void mma_tile_regs(v16f (&acc)[2], const float *tile, const float (&f)[32], int lr, int lk) {
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nb][r] = 0.0f;
    const float *ap = tile + (nb * 32 + lr) * kLd + lk * 32;
#pragma unroll
    for (int i4 = 0; i4 < 8; ++i4) {
      const v4f a = *reinterpret_cast<const v4f *>(ap + 4 * i4);
      acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, f[4 * i4], acc[nb], 0, 0, 0);
      acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, f[4 * i4 + 1], acc[nb], 0, 0, 0);
      acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, f[4 * i4 + 2], acc[nb], 0, 0, 0);
      acc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, f[4 * i4 + 3], acc[nb], 0, 0, 0);
    }
  }
}

// acc^T (64 head columns x 32) += tile^T x, contracting the 64 tile rows: step (nb, r) pairs the rows
// 32 nb + 8 (r / 4) + r % 4 (lk = 0) and that + 4 (lk = 1), which is where x[nb][r] sits in an accumulator
__device__ __forceinline__ void mma_tileT_acc(v16f (&acc)[2], const float *tile, const v16f (&x)[2], int lr, int lk) {
  const int col = parity_major(lr);
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float *ap = tile + (32 * nb + 8 * (r >> 2) + 4 * lk + (r & 3)) * kLd + col;
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[0], x[nb][r], acc[0], 0, 0, 0);
      acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[16], x[nb][r], acc[1], 0, 0, 0);
    }
}

// a wavefront's 64 x 32 transposed result out through its quarter of the LDS block as whole rows of `out`
__device__ __forceinline__ void store_rows(float *ot, const v16f (&acc)[2], float mul, float *__restrict__ out,
                                           int64_t ld_out, int64_t row0, int64_t rows, int dh, int lane, int lr, int lk) {
#pragma unroll
  for (int blk = 0; blk < 2; ++blk)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      v4f v;
      v.x = acc[blk][4 * r4] * mul; v.y = acc[blk][4 * r4 + 1] * mul;
      v.z = acc[blk][4 * r4 + 2] * mul; v.w = acc[blk][4 * r4 + 3] * mul;
      *reinterpret_cast<v4f *>(ot + lr * kLd + 32 * blk + 8 * r4 + 4 * lk) = v;
    }
  __builtin_amdgcn_wave_barrier();
  for (int q = 0; q < 32; ++q)
    if (row0 + q < rows && lane < dh) out[(row0 + q) * ld_out + lane] = ot[q * kLd + lane];
  __builtin_amdgcn_wave_barrier();
}

__global__ __launch_bounds__(kThreads) void attention_bwd_dq_kernel(const float *__restrict__ qkv,
                                                                    const float *__restrict__ dctx,
                                                                    const float *__restrict__ lse,
                                                                    const float *__restrict__ dsum, AttnGeom g,
                                                                    float *__restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) float lds[2 * kK * kLd];
  float *Kp = lds, *Vp = lds + kK * kLd;   // keys and values, both parity-major along the head
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lk = lane >> 5;
  int64_t id = blockIdx.x;
  const int qt = static_cast<int>(id % g.qtiles);
  id /= g.qtiles;
  const int h = static_cast<int>(id % g.heads);
  const int64_t b = id / g.heads;
  const int64_t t0 = static_cast<int64_t>(qt) * kQ;
  const int64_t hc = static_cast<int64_t>(h) * g.dh;
  float qf[32], dof[32];
  stage_tile(Kp, qkv, 3 * g.D, g, b, t0, hc, true);
  stage_tile(Vp, qkv, 3 * g.D, g, b, t0 + 64, hc, true);
  __syncthreads();
  take_rows(qf, Kp, Vp, wave, lr, lk);
  __syncthreads();
  stage_tile(Kp, dctx, g.D, g, b, t0, hc, true);
  stage_tile(Vp, dctx, g.D, g, b, t0 + 64, hc, true);
  __syncthreads();
  take_rows(dof, Kp, Vp, wave, lr, lk);
  const int64_t tw = t0 + wave * 32;
  const bool active = tw < g.T;
  const int64_t t = tw + lr, tc = t < g.T ? t : g.T - 1;
  const float L = lse[(b * g.T + tc) * g.heads + h], Dt = dsum[(b * g.T + tc) * g.heads + h];
  const int64_t tlast = (t0 + kQ - 1 < g.T ? t0 + kQ - 1 : g.T - 1);
  const int64_t jmin = (g.left < 0 || t0 - g.left < 0) ? 0 : t0 - g.left;
  const int64_t jmax = (g.right < 0 || tlast + g.right > g.T - 1) ? g.T - 1 : tlast + g.right;
  const int64_t wlo = g.left < 0 ? 0 : t - g.left;
  const int64_t whi = (g.right < 0 || t + g.right > g.T - 1) ? g.T - 1 : t + g.right;
  v16f dq[2];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    dq[0][r] = 0.0f;
    dq[1][r] = 0.0f;
  }
  float kn[16], vn[16];   // keys and values of the next step, in flight while this step computes
  const int64_t jfirst = jmin / kK * kK;
  load_tile(kn, qkv, 3 * g.D, g, b, jfirst, g.D + hc);
  load_tile(vn, qkv, 3 * g.D, g, b, jfirst, 2 * g.D + hc);
  for (int64_t j0 = jfirst; j0 <= jmax; j0 += kK) {
    __syncthreads();
    store_tile(Kp, kn, g, j0, true);
    store_tile(Vp, vn, g, j0, true);
    __syncthreads();
    if (j0 + kK <= jmax) {
      load_tile(kn, qkv, 3 * g.D, g, b, j0 + kK, g.D + hc);
      load_tile(vn, qkv, 3 * g.D, g, b, j0 + kK, 2 * g.D + hc);
    }
    if (active) {
      v16f s[2], dp[2];
      mma_tile_regs(s, Kp, qf, lr, lk);     // S^T: keys x this lane's query
      mma_tile_regs(dp, Vp, dof, lr, lk);   // dP^T
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t j = j0 + 32 * nb + 8 * (r >> 2) + 4 * lk + (r & 3);
          const float p = (j >= wlo && j <= whi) ? __builtin_amdgcn_exp2f(s[nb][r] * g.scale_log2e - L) : 0.0f;
          s[nb][r] = p * (dp[nb][r] - Dt);
        }
      mma_tileT_acc(dq, Kp, s, lr, lk);     // dQ^T += K^T dS^T
    }
  }
  __syncthreads();
  if (active)
    store_rows(lds + wave * 32 * kLd, dq, g.scale, dqkv + b * g.T * 3 * g.D + hc, 3 * g.D, tw, g.T, g.dh, lane, lr, lk);
}

__global__ __launch_bounds__(kThreads) void attention_bwd_dkv_kernel(const float *__restrict__ qkv,
                                                                     const float *__restrict__ dctx,
                                                                     const float *__restrict__ lse,
                                                                     const float *__restrict__ dsum, AttnGeom g,
                                                                     float *__restrict__ dqkv) {
  __shared__ __attribute__((aligned(16))) float lds[2 * kK * kLd];
  __shared__ float Ls[kK], Ds[kK];
  float *Qp = lds, *Gp = lds + kK * kLd;   // queries and upstream gradient rows, both parity-major along the head
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lr = lane & 31, lk = lane >> 5;
  int64_t id = blockIdx.x;
  const int kt = static_cast<int>(id % g.qtiles);
  id /= g.qtiles;
  const int h = static_cast<int>(id % g.heads);
  const int64_t b = id / g.heads;
  const int64_t j0t = static_cast<int64_t>(kt) * kQ;
  const int64_t hc = static_cast<int64_t>(h) * g.dh;
  float kf[32], vf[32];
  stage_tile(Qp, qkv, 3 * g.D, g, b, j0t, g.D + hc, true);
  stage_tile(Gp, qkv, 3 * g.D, g, b, j0t + 64, g.D + hc, true);
  __syncthreads();
  take_rows(kf, Qp, Gp, wave, lr, lk);
  __syncthreads();
  stage_tile(Qp, qkv, 3 * g.D, g, b, j0t, 2 * g.D + hc, true);
  stage_tile(Gp, qkv, 3 * g.D, g, b, j0t + 64, 2 * g.D + hc, true);
  __syncthreads();
  take_rows(vf, Qp, Gp, wave, lr, lk);
  const int64_t jw = j0t + wave * 32;
  const bool active = jw < g.T;
  const int64_t j = jw + lr;                 // this lane's key frame
  // query frames that may look at a key of this tile
  const int64_t jlast = (j0t + kQ - 1 < g.T ? j0t + kQ - 1 : g.T - 1);
  const int64_t tmin = (g.right < 0 || j0t - g.right < 0) ? 0 : j0t - g.right;
  const int64_t tmax = (g.left < 0 || jlast + g.left > g.T - 1) ? g.T - 1 : jlast + g.left;
  // the queries t with t - left <= j <= t + right
  const int64_t qlo = g.right < 0 ? 0 : j - g.right;
  const int64_t qhi = (g.left < 0 || j + g.left > g.T - 1) ? g.T - 1 : j + g.left;
  v16f dk[2], dv[2];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    dk[0][r] = 0.0f; dk[1][r] = 0.0f;
    dv[0][r] = 0.0f; dv[1][r] = 0.0f;
  }
  float qn[16], gn[16];   // queries and upstream gradient rows of the next step, in flight while this step computes
  const int64_t tfirst = tmin / kK * kK;
  load_tile(qn, qkv, 3 * g.D, g, b, tfirst, hc);
  load_tile(gn, dctx, g.D, g, b, tfirst, hc);
  for (int64_t tq = tfirst; tq <= tmax; tq += kK) {
    __syncthreads();
    store_tile(Qp, qn, g, tq, true);
    store_tile(Gp, gn, g, tq, true);
    if (tid < kK) {
      const int64_t tt = tq + tid < g.T ? tq + tid : g.T - 1;
      Ls[tid] = lse[(b * g.T + tt) * g.heads + h];
      Ds[tid] = dsum[(b * g.T + tt) * g.heads + h];
    }
    __syncthreads();
    if (tq + kK <= tmax) {
      load_tile(qn, qkv, 3 * g.D, g, b, tq + kK, hc);
      load_tile(gn, dctx, g.D, g, b, tq + kK, hc);
    }
    if (active) {
      v16f s[2], dp[2];
      mma_tile_regs(s, Qp, kf, lr, lk);     // S: queries x this lane's key
      mma_tile_regs(dp, Gp, vf, lr, lk);    // dP
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 32 * nb + 8 * (r >> 2) + 4 * lk + (r & 3);
          const int64_t tt = tq + row;
          const float p = (j < g.T && tt >= qlo && tt <= qhi) ? __builtin_amdgcn_exp2f(s[nb][r] * g.scale_log2e - Ls[row]) : 0.0f;
          s[nb][r] = p;
          dp[nb][r] = p * (dp[nb][r] - Ds[row]);
        }
      mma_tileT_acc(dv, Gp, s, lr, lk);     // dV^T += dO^T P
      mma_tileT_acc(dk, Qp, dp, lr, lk);    // dK^T += Q^T dS
    }
  }
  __syncthreads();
  if (active) {
    float *ot = lds + wave * 32 * kLd;
    store_rows(ot, dk, g.scale, dqkv + b * g.T * 3 * g.D + g.D + hc, 3 * g.D, jw, g.T, g.dh, lane, lr, lk);
    store_rows(ot, dv, 1.0f, dqkv + b * g.T * 3 * g.D + 2 * g.D + hc, 3 * g.D, jw, g.T, g.dh, lane, lr, lk);
  }
}

__global__ void zero_attn_absmax_kernel(uint32_t *p) {
  if (threadIdx.x == 0) *p = 0u;
}

AttnGeom attn_geom(int64_t B, int64_t T, int64_t D, int heads, int left, int right) {
  AttnGeom g;
  g.B = B; g.T = T; g.D = D; g.heads = heads; g.dh = static_cast<int>(D / heads);
  g.left = left; g.right = right;
  g.qtiles = static_cast<int>(cdiv(T, kQ));
  g.scale_log2e = static_cast<float>(1.4426950408889634 / sqrt(static_cast<double>(g.dh)));
  g.scale = static_cast<float>(1.0 / sqrt(static_cast<double>(g.dh)));
  return g;
}

}  // namespace

bool attention_shape_ok(int64_t B, int64_t T, int64_t D, int heads) {
  if (B < 1 || T < 1 || D < 1 || heads < 1 || D % heads) return false;
  const int64_t dh = D / heads;
  if (dh > kDh) return false;
  return cdiv(T, kQ) * heads <= (int64_t(1) << 31) / B - 1;
}

aqt_status launch_attention(const float *qkv, int64_t B, int64_t T, int64_t D, int heads, int left, int right,
                            float *ctx, uint32_t *absmax, float *lse, hipStream_t st, bool absmax_is_zero) {
  const AttnGeom g = attn_geom(B, T, D, heads, left, right);
  if (absmax && !absmax_is_zero) zero_attn_absmax_kernel<<<1, 64, 0, st>>>(absmax);
  const int64_t blocks = static_cast<int64_t>(g.qtiles) * heads * B;
  attention_fwd_kernel<<<static_cast<unsigned>(blocks), kThreads, 0, st>>>(qkv, g, ctx, absmax, lse);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

size_t attention_bwd_ws_bytes(int64_t B, int64_t T, int heads) {
  return align_up(static_cast<size_t>(B) * T * heads * sizeof(float), 256);
}

aqt_status launch_attention_bwd(const float *qkv, const float *ctx, const float *dctx, const float *lse, int64_t B,
                                int64_t T, int64_t D, int heads, int left, int right, float *dqkv, void *ws,
                                hipStream_t st) {
  const AttnGeom g = attn_geom(B, T, D, heads, left, right);
  float *dsum = static_cast<float *>(ws);
  int64_t rg = cdiv(B * T, 4);
  if (rg > 4096) rg = 4096;
  attention_rowdot_kernel<<<static_cast<unsigned>(rg), kThreads, 0, st>>>(dctx, ctx, g, dsum);
  AQT_HIP(hipGetLastError());
  const unsigned blocks = static_cast<unsigned>(static_cast<int64_t>(g.qtiles) * heads * B);
  attention_bwd_dq_kernel<<<blocks, kThreads, 0, st>>>(qkv, dctx, lse, dsum, g, dqkv);
  AQT_HIP(hipGetLastError());
  attention_bwd_dkv_kernel<<<blocks, kThreads, 0, st>>>(qkv, dctx, lse, dsum, g, dqkv);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
