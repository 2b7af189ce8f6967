// The float core of the Conformer self-attention module between its two quantized
// projections (arxiv 2203.15952, Sec. 3.2: 4 or 8 heads; Sec. 3.3: a limited left context
// and, in the non-causal encoder, a limited right context): for every utterance, head and
// query frame, softmax over the key frames of the window of the scaled dot products, times
// the values.  Plain float32 vector arithmetic with an online softmax (running maximum and
// sum per query, the output rescaled when the maximum moves), so the scores never leave the
// chip; the largest |result| is reduced on the way out for the quantizer of the output
// projection (Fig. 2).
//
// qkv [B*T, 3D]: queries, keys, values in three column blocks of width D, head h in columns
// h*dh .. (h+1)*dh of each.  A workgroup owns 64 query frames of one utterance and head and
// walks the key frames of their windows 64 at a time: queries, keys and values sit in LDS
// (rows of 68 floats: 16-byte aligned and conflict-free for the access patterns below), a
// thread forms 4 x 4 blocks: queries 4 ty .. 4 ty + 3 against keys tx, tx + 16, tx + 32,
// tx + 48 for the scores, the same queries against head columns 4 tx .. 4 tx + 3 for the
// output.  The probabilities pass through the LDS block the keys held.
#include "aqt_internal.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;
constexpr int kQ = 64;          // query frames per workgroup
constexpr int kK = 64;          // key frames per step
constexpr int kDh = 64;         // widest head a tile holds; narrower heads are padded with zeros
constexpr int kLd = kDh + 4;    // LDS row stride in floats
typedef float v4f __attribute__((ext_vector_type(4)));

struct AttnGeom {
  int64_t B, T, D;
  int heads, dh, left, right;   // left / right < 0: no limit on that side
  int qtiles;                   // 64-frame query tiles per utterance
  float scale;                  // 1 / sqrt(dh)
};

__device__ __forceinline__ float group16_max(float v) {
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float group16_sum(float v) {
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ uint32_t wave_max_bits(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), off, 64));
    v = v > o ? v : o;
  }
  return v;
}

// 64 frames x 64 head columns starting at frame row0 and qkv column col0 into dst[frame][col]; frames
// beyond the utterance and columns beyond the head are zero.  Loads go to clamped, always valid
// addresses (no branches, sixteen in flight per thread).
__device__ __forceinline__ void stage_tile(float *__restrict__ dst, const float *__restrict__ qkv, const AttnGeom &g,
                                           int64_t b, int64_t row0, int64_t col0) {
  const int d = threadIdx.x & 63, r0 = threadIdx.x >> 6;
  const int dd = d < g.dh ? d : g.dh - 1;
  float v[16];
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    int64_t t = row0 + r0 + 4 * k;
    t = t < g.T ? t : g.T - 1;
    v[k] = qkv[(b * g.T + t) * 3 * g.D + col0 + dd];
  }
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int r = r0 + 4 * k;
    dst[r * kLd + d] = (d < g.dh && row0 + r < g.T) ? v[k] : 0.0f;
  }
}

__global__ __launch_bounds__(kThreads) void attention_fwd_kernel(const float *__restrict__ qkv, AttnGeom g,
                                                                 float *__restrict__ ctx,
                                                                 uint32_t *__restrict__ absmax) {
  __shared__ float Qs[kQ * kLd];
  __shared__ float Ks[kK * kLd];   // keys, then the probabilities of the same step
  __shared__ float Vs[kK * kLd];
  float *Ps = Ks;
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  int64_t id = blockIdx.x;
  const int qt = static_cast<int>(id % g.qtiles);
  id /= g.qtiles;
  const int h = static_cast<int>(id % g.heads);
  const int64_t b = id / g.heads;
  const int64_t t0 = static_cast<int64_t>(qt) * kQ;
  const int64_t hc = static_cast<int64_t>(h) * g.dh;
  stage_tile(Qs, qkv, g, b, t0, hc);

  // key frames any query of this tile may look at
  const int64_t tlast = (t0 + kQ - 1 < g.T ? t0 + kQ - 1 : g.T - 1);
  const int64_t jmin = (g.left < 0 || t0 - g.left < 0) ? 0 : t0 - g.left;
  const int64_t jmax = (g.right < 0 || tlast + g.right > g.T - 1) ? g.T - 1 : tlast + g.right;

  float m[4], l[4], o[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    m[i] = -1e30f;
    l[i] = 0.0f;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[i][e] = 0.0f;
  }
  for (int64_t j0 = jmin / kK * kK; j0 <= jmax; j0 += kK) {
    __syncthreads();   // the previous step's reads of Ps and Vs are over (first step: Qs is complete after the next barrier)
    stage_tile(Ks, qkv, g, b, j0, g.D + hc);
    stage_tile(Vs, qkv, g, b, j0, 2 * g.D + hc);
    __syncthreads();
    // scores of queries 4 ty + i against keys tx + 16 kk
    float s[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) s[i][kk] = 0.0f;
#pragma unroll 4
    for (int d4 = 0; d4 < kDh; d4 += 4) {
      v4f q[4], k[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) q[i] = *reinterpret_cast<const v4f *>(&Qs[(ty * 4 + i) * kLd + d4]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) k[kk] = *reinterpret_cast<const v4f *>(&Ks[(tx + 16 * kk) * kLd + d4]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          s[i][kk] = fmaf(q[i].x, k[kk].x, s[i][kk]);
          s[i][kk] = fmaf(q[i].y, k[kk].y, s[i][kk]);
          s[i][kk] = fmaf(q[i].z, k[kk].z, s[i][kk]);
          s[i][kk] = fmaf(q[i].w, k[kk].w, s[i][kk]);
        }
    }
    // window, running maximum and sum, probabilities
    float alpha[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int64_t t = t0 + ty * 4 + i;
      bool ok[4];
      float mx = -1e30f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int64_t j = j0 + tx + 16 * kk;
        ok[kk] = j < g.T && (g.left < 0 || j >= t - g.left) && (g.right < 0 || j <= t + g.right);
        s[i][kk] *= g.scale;
        if (ok[kk]) mx = fmaxf(mx, s[i][kk]);
      }
      const float mnew = fmaxf(m[i], group16_max(mx));
      alpha[i] = expf(m[i] - mnew);
      float sum = 0.0f;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s[i][kk] = ok[kk] ? expf(s[i][kk] - mnew) : 0.0f;
        sum += s[i][kk];
      }
      l[i] = l[i] * alpha[i] + group16_sum(sum);
      m[i] = mnew;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[i][e] *= alpha[i];
    }
    __syncthreads();   // every score has been formed: the keys may be overwritten
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) Ps[(ty * 4 + i) * kLd + tx + 16 * kk] = s[i][kk];
    __syncthreads();
    // output columns 4 tx .. 4 tx + 3 of queries 4 ty + i
#pragma unroll 4
    for (int j4 = 0; j4 < kK; j4 += 4) {
      v4f p[4], v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) p[i] = *reinterpret_cast<const v4f *>(&Ps[(ty * 4 + i) * kLd + j4]);
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) v[jj] = *reinterpret_cast<const v4f *>(&Vs[(j4 + jj) * kLd + tx * 4]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        o[i][0] = fmaf(p[i].x, v[0].x, o[i][0]); o[i][1] = fmaf(p[i].x, v[0].y, o[i][1]);
        o[i][2] = fmaf(p[i].x, v[0].z, o[i][2]); o[i][3] = fmaf(p[i].x, v[0].w, o[i][3]);
        o[i][0] = fmaf(p[i].y, v[1].x, o[i][0]); o[i][1] = fmaf(p[i].y, v[1].y, o[i][1]);
        o[i][2] = fmaf(p[i].y, v[1].z, o[i][2]); o[i][3] = fmaf(p[i].y, v[1].w, o[i][3]);
        o[i][0] = fmaf(p[i].z, v[2].x, o[i][0]); o[i][1] = fmaf(p[i].z, v[2].y, o[i][1]);
        o[i][2] = fmaf(p[i].z, v[2].z, o[i][2]); o[i][3] = fmaf(p[i].z, v[2].w, o[i][3]);
        o[i][0] = fmaf(p[i].w, v[3].x, o[i][0]); o[i][1] = fmaf(p[i].w, v[3].y, o[i][1]);
        o[i][2] = fmaf(p[i].w, v[3].z, o[i][2]); o[i][3] = fmaf(p[i].w, v[3].w, o[i][3]);
      }
    }
  }
  uint32_t amax = 0u;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t t = t0 + ty * 4 + i;
    if (t < g.T) {
      const float inv = l[i] > 0.0f ? 1.0f / l[i] : 0.0f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int d = tx * 4 + e;
        if (d < g.dh) {
          const float r = o[i][e] * inv;
          ctx[(b * g.T + t) * g.D + hc + d] = r;
          amax = max(amax, __float_as_uint(r) & 0x7FFFFFFFu);
        }
      }
    }
  }
  if (absmax) {   // uniform: the word only grows, so a stale read can only cost a redundant atomic
    amax = wave_max_bits(amax);
    if ((tid & 63) == 0 && amax > *reinterpret_cast<volatile uint32_t *>(absmax)) atomicMax(absmax, amax);
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
  g.scale = 1.0f / sqrtf(static_cast<float>(g.dh));
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
                            float *ctx, uint32_t *absmax, hipStream_t st) {
  const AttnGeom g = attn_geom(B, T, D, heads, left, right);
  if (absmax) zero_attn_absmax_kernel<<<1, 64, 0, st>>>(absmax);
  const int64_t blocks = static_cast<int64_t>(g.qtiles) * heads * B;
  attention_fwd_kernel<<<static_cast<unsigned>(blocks), kThreads, 0, st>>>(qkv, g, ctx, absmax);
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace aqt
