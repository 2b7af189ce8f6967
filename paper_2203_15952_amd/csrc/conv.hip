// The float layers between the two pointwise convolutions of the Conformer convolution
// module (arxiv 2203.15952, Sec. 3.2: depthwise kernel size 32; Sec. 3.3: causal depthwise
// convolution of kernel size 15, and convolution kernels are left unquantized): depthwise
// convolution along time, the normalisation behind it with fixed statistics (one scale and
// one shift per channel), Swish, and the abs-max of the result for the quantizer of the
// second pointwise convolution (Fig. 2), in one pass over the tensor; the adjoint kernels
// for the backward.  Plain float32 vector arithmetic: about 32 multiply-adds per 8 bytes
// moved, so HBM time bounds these kernels, not the ALUs.
//
// Layout: x [B,T,C], C contiguous (tokens x channels, B utterances of T frames); w [kw,C].
// A workgroup owns 64 frames x 64 channels of one utterance: the frames it needs (64 + kw - 1
// rows, each a coalesced 256-byte piece per wavefront) and the taps go to LDS once, a lane
// owns a channel (LDS reads are conflict-free) and forms four neighbouring results at a time
// from a sliding window of four values, one LDS read per tap for the values and one for the
// tap.  Neighbouring tiles share their halo through L2.
#include "aqt_internal.h"
#include "epilogue.h"

namespace aqt {
namespace {

constexpr int kThreads = 256;
constexpr int kTile = 64;      // frames per workgroup tile
constexpr int kTapsMax = 32;   // largest kernel size the tiled kernels take (at most 198 LDS rows of 256 bytes)

__device__ __forceinline__ uint32_t wave_max_bits(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const uint32_t o = static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), off, 64));
    v = v > o ? v : o;
  }
  return v;
}

struct ConvGeom {
  int64_t B, T, C;
  int kw, pad_left;
  int cgroups, tgroups;   // 64-channel groups; 64-frame tiles per utterance
};

// Stage rows [t0 - pl, t0 - pl + rows) of channel group cg of utterance b into LDS as
// xs[row][lane] (zero outside the utterance and beyond channel C), multiplied by xmul if given.
// Eight rows per wavefront are in flight at a time: every load goes to a clamped, always valid
// address and the value is zeroed afterwards, so the loads carry no branches and overlap.
__device__ __forceinline__ void stage_frames(float *__restrict__ xs, int rows, const float *__restrict__ xin,
                                             const float *__restrict__ xmul, const ConvGeom &g, int64_t b,
                                             int64_t t0, int pl, int64_t c) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t cc = c < g.C ? c : g.C - 1;
  const float *xb = xin + b * g.T * g.C + cc;
  const float *mb = xmul ? xmul + b * g.T * g.C + cc : nullptr;
  for (int r0 = wave; r0 < rows; r0 += 32) {
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      int64_t tt = t0 + (r0 + 4 * k) - pl;
      tt = tt < 0 ? 0 : (tt >= g.T ? g.T - 1 : tt);
      v[k] = xb[tt * g.C];
    }
    if (mb) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        int64_t tt = t0 + (r0 + 4 * k) - pl;
        tt = tt < 0 ? 0 : (tt >= g.T ? g.T - 1 : tt);
        v[k] *= mb[tt * g.C];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int r = r0 + 4 * k;
      const int64_t tt = t0 + r - pl;
      if (r < rows) xs[r * 64 + lane] = (c < g.C && tt >= 0 && tt < g.T) ? v[k] : 0.0f;
    }
  }
}

// out[b,t,c] = act( (bias[c] + sum_j tap_j * in[b, t + j - pl, c]) * na[c] + nb[c] ),  in = xin (* xmul)
// tap_j = w[j] (the layer itself), or w[kw - 1 - j] when rev (the gradient with respect to the
// input is the correlation of the upstream gradient with the mirrored kernel, and the caller
// passes pl = kw - 1 - pad_left).  dfac (nullable) receives d out / d (convolution result);
// absmax (nullable) the largest |out| as float bits.  Dynamic LDS: (kTile + 2 kw - 1) * 256 bytes.
__global__ __launch_bounds__(kThreads) void dwconv_kernel(const float *__restrict__ xin, const float *__restrict__ xmul,
                                                          const float *__restrict__ w, const float *__restrict__ bias,
                                                          const float *__restrict__ na, const float *__restrict__ nb,
                                                          int swish, int rev, ConvGeom g, int pl,
                                                          float *__restrict__ out, float *__restrict__ dfac,
                                                          uint32_t *__restrict__ absmax) {
  extern __shared__ float lds[];
  const int rows = kTile + g.kw - 1;
  float *xs = lds;               // [rows][64]
  float *ws = lds + rows * 64;   // [kw][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t id = blockIdx.x;
  const int cg = static_cast<int>(id % g.cgroups);
  id /= g.cgroups;
  const int tg = static_cast<int>(id % g.tgroups);
  const int64_t b = id / g.tgroups;
  const int64_t c = static_cast<int64_t>(cg) * 64 + lane;
  const int64_t t0 = static_cast<int64_t>(tg) * kTile;
  stage_frames(xs, rows, xin, xmul, g, b, t0, pl, c);
  for (int j = wave; j < g.kw; j += 4)
    ws[j * 64 + lane] = (c < g.C) ? w[static_cast<int64_t>(rev ? g.kw - 1 - j : j) * g.C + c] : 0.0f;
  __syncthreads();
  uint32_t amax = 0u;
  if (c < g.C) {
    const float b0 = bias ? bias[c] : 0.0f;
    const float a = na ? na[c] : 1.0f, sh = nb ? nb[c] : 0.0f;
    for (int grp = 0; grp < 4; ++grp) {
      const int tl = wave * 16 + grp * 4;
      if (t0 + tl >= g.T) break;
      float acc[4] = {b0, b0, b0, b0};
      float x0 = xs[tl * 64 + lane], x1 = xs[(tl + 1) * 64 + lane], x2 = xs[(tl + 2) * 64 + lane];
#pragma unroll 8
      for (int j = 0; j < g.kw; ++j) {
        const float x3 = xs[(tl + j + 3) * 64 + lane];
        const float wj = ws[j * 64 + lane];
        acc[0] = fmaf(wj, x0, acc[0]);
        acc[1] = fmaf(wj, x1, acc[1]);
        acc[2] = fmaf(wj, x2, acc[2]);
        acc[3] = fmaf(wj, x3, acc[3]);
        x0 = x1;
        x1 = x2;
        x2 = x3;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int64_t t = t0 + tl + k;
        if (t < g.T) {
          float n = acc[k];
          if (na) n = n * a;
          if (nb) n = n + sh;
          float o = n, df = a;
          if (swish) {
            const float sg = sigmoid_f32(n);
            o = n * sg;
            df = a * swish_dact_f32(n, sg);
          }
          const int64_t at = (b * g.T + t) * g.C + c;
          out[at] = o;
          if (dfac) dfac[at] = df;
          amax = max(amax, __float_as_uint(o) & 0x7FFFFFFFu);
        }
      }
    }
  }
  if (absmax) {   // uniform: the word only grows, so a stale read can only cost a redundant atomic
    amax = wave_max_bits(amax);
    if (lane == 0 && amax > *reinterpret_cast<volatile uint32_t *>(absmax)) atomicMax(absmax, amax);
  }
}

// Any kernel size: one thread per output element.
__global__ __launch_bounds__(kThreads) void dwconv_any_kernel(const float *__restrict__ xin,
                                                              const float *__restrict__ xmul,
                                                              const float *__restrict__ w, const float *__restrict__ bias,
                                                              const float *__restrict__ na, const float *__restrict__ nb,
                                                              int swish, int rev, ConvGeom g, int pl,
                                                              float *__restrict__ out, float *__restrict__ dfac,
                                                              uint32_t *__restrict__ absmax) {
  const int64_t total = g.B * g.T * g.C;
  const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
  uint32_t amax = 0u;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < total; i += stride) {
    const int64_t c = i % g.C, bt = i / g.C, t = bt % g.T, b = bt / g.T;
    float acc = bias ? bias[c] : 0.0f;
    for (int j = 0; j < g.kw; ++j) {
      const int64_t tt = t + j - pl;
      if (tt < 0 || tt >= g.T) continue;
      const int64_t at = (b * g.T + tt) * g.C + c;
      float xv = xin[at];
      if (xmul) xv *= xmul[at];
      acc = fmaf(w[static_cast<int64_t>(rev ? g.kw - 1 - j : j) * g.C + c], xv, acc);
    }
    const float a = na ? na[c] : 1.0f;
    float n = acc;
    if (na) n = n * a;
    if (nb) n = n + nb[c];
    float o = n, df = a;
    if (swish) {
      const float sg = sigmoid_f32(n);
      o = n * sg;
      df = a * swish_dact_f32(n, sg);
    }
    out[i] = o;
    if (dfac) dfac[i] = df;
    amax = max(amax, __float_as_uint(o) & 0x7FFFFFFFu);
  }
  if (absmax) {
    amax = wave_max_bits(amax);
    if ((threadIdx.x & 63) == 0 && amax > *reinterpret_cast<volatile uint32_t *>(absmax)) atomicMax(absmax, amax);
  }
}

__global__ void zero_absmax_kernel(uint32_t *p) {
  if (threadIdx.x == 0) *p = 0u;
}

// Gradient of the taps and of the bias:
//   dw[j,c] = sum_{b,t} dv[b,t,c] * x[b, t + j - pl, c],   dbias[c] = sum_{b,t} dv[b,t,c],   dv = dout (* dmul).
// Workgroup (cg, p) walks the tiles p, p + P, ... of its 64-channel group (a tile = 64 frames of
// one utterance): dv and the frames of x it meets go to LDS; a lane owns a channel, a wavefront
// owns groups of four neighbouring taps and adds its tile sums into LDS accumulators only it
// touches.  The workgroup leaves one partial per tap and channel; dwconv_dw_fold_kernel adds the
// P partials in order.  Same bits on every run.
// Dynamic LDS: (2 kTile + kw + 2) + (kwp + 4) rows of 256 bytes, kwp = kw rounded up to 4.
__global__ __launch_bounds__(kThreads) void dwconv_dw_kernel(const float *__restrict__ dout,
                                                             const float *__restrict__ dmul,
                                                             const float *__restrict__ x, ConvGeom g, int P,
                                                             float *__restrict__ part) {
  extern __shared__ float lds[];
  const int kwp = (g.kw + 3) & ~3;
  const int rows = kTile + kwp + 2;             // frames of x a tile meets, incl. the window's run-out
  float *dvs = lds;                             // [kTile][64]
  float *xs = dvs + kTile * 64;                 // [rows][64]
  float *accw = xs + rows * 64;                 // [kwp][64] tap sums
  float *accb = accw + kwp * 64;                // [4][64]   bias sums, one row per wavefront
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int cg = blockIdx.x % g.cgroups, p = blockIdx.x / g.cgroups;
  const int64_t c = static_cast<int64_t>(cg) * 64 + lane;
  for (int j = wave; j < kwp + 4; j += 4) accw[j * 64 + lane] = 0.0f;   // accb follows accw
  const int64_t ntile = g.B * g.tgroups;
  for (int64_t q = p; q < ntile; q += P) {
    const int64_t b = q / g.tgroups;
    const int64_t t0 = (q % g.tgroups) * kTile;
    __syncthreads();   // the previous tile's reads are over
    stage_frames(dvs, kTile, dout, dmul, g, b, t0, 0, c);
    stage_frames(xs, rows, x, nullptr, g, b, t0, g.pad_left, c);
    __syncthreads();
    float sb = 0.0f;
    for (int t = wave * 16; t < wave * 16 + 16; ++t) sb += dvs[t * 64 + lane];
    accb[wave * 64 + lane] += sb;
    for (int j0 = wave * 4; j0 < g.kw; j0 += 16) {
      float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
      float x0 = xs[j0 * 64 + lane], x1 = xs[(j0 + 1) * 64 + lane], x2 = xs[(j0 + 2) * 64 + lane];
#pragma unroll 8
      for (int t = 0; t < kTile; ++t) {
        const float x3 = xs[(t + j0 + 3) * 64 + lane];
        const float d = dvs[t * 64 + lane];
        a0 = fmaf(d, x0, a0);
        a1 = fmaf(d, x1, a1);
        a2 = fmaf(d, x2, a2);
        a3 = fmaf(d, x3, a3);
        x0 = x1;
        x1 = x2;
        x2 = x3;
      }
      accw[j0 * 64 + lane] += a0;
      accw[(j0 + 1) * 64 + lane] += a1;
      accw[(j0 + 2) * 64 + lane] += a2;
      accw[(j0 + 3) * 64 + lane] += a3;
    }
  }
  __syncthreads();
  if (c < g.C) {
    float *o = part + static_cast<int64_t>(p) * (g.kw + 1) * g.C + c;
    for (int j = wave; j < g.kw; j += 4) o[static_cast<int64_t>(j) * g.C] = accw[j * 64 + lane];
    if (wave == 0)
      o[static_cast<int64_t>(g.kw) * g.C] =
          ((accb[lane] + accb[64 + lane]) + accb[128 + lane]) + accb[192 + lane];   // the bias sum sits behind the taps
  }
}

// Any kernel size: one thread per (tap, channel), the whole sum over (b, t) in order; the
// bias sum is row kw.  P = 1.
__global__ __launch_bounds__(kThreads) void dwconv_dw_any_kernel(const float *__restrict__ dout,
                                                                 const float *__restrict__ dmul,
                                                                 const float *__restrict__ x, ConvGeom g,
                                                                 float *__restrict__ part) {
  const int64_t total = static_cast<int64_t>(g.kw + 1) * g.C;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i >= total) return;
  const int64_t c = i % g.C;
  const int j = static_cast<int>(i / g.C);
  float acc = 0.0f;
  for (int64_t b = 0; b < g.B; ++b)
    for (int64_t t = 0; t < g.T; ++t) {
      const int64_t at = (b * g.T + t) * g.C + c;
      float v = dout[at];
      if (dmul) v *= dmul[at];
      if (j == g.kw) {
        acc += v;
      } else {
        const int64_t tt = t + j - g.pad_left;
        if (tt >= 0 && tt < g.T) acc = fmaf(v, x[(b * g.T + tt) * g.C + c], acc);
      }
    }
  part[i] = acc;
}

__global__ __launch_bounds__(kThreads) void dwconv_dw_fold_kernel(const float *__restrict__ part, int P, int kw,
                                                                  int64_t C, float *__restrict__ dw,
                                                                  float *__restrict__ dbias) {
  const int64_t rows = kw + 1;
  const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (i >= rows * C) return;
  // four independent running sums (partials p = 0, 4, 8, ...; 1, 5, ...; ...) so that loads overlap; the order
  // of the additions is fixed all the same
  float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
  int p = 0;
  for (; p + 4 <= P; p += 4) {
    s0 += part[static_cast<int64_t>(p) * rows * C + i];
    s1 += part[static_cast<int64_t>(p + 1) * rows * C + i];
    s2 += part[static_cast<int64_t>(p + 2) * rows * C + i];
    s3 += part[static_cast<int64_t>(p + 3) * rows * C + i];
  }
  for (; p < P; ++p) s0 += part[static_cast<int64_t>(p) * rows * C + i];
  const float s = (s0 + s1) + (s2 + s3);
  if (i < static_cast<int64_t>(kw) * C) {
    if (dw) dw[i] = s;
  } else if (dbias) {
    dbias[i - static_cast<int64_t>(kw) * C] = s;
  }
}

ConvGeom geom(int64_t B, int64_t T, int64_t C, int kw, int pad_left) {
  ConvGeom g;
  g.B = B; g.T = T; g.C = C; g.kw = kw; g.pad_left = pad_left;
  g.cgroups = static_cast<int>(cdiv(C, 64));
  g.tgroups = static_cast<int>(cdiv(T, kTile));
  return g;
}

// Partials of the tap gradient: as many workgroups per channel group as give the chip a few
// workgroups per compute unit, never more than there are tiles.
int dw_partials(const ConvGeom &g) {
  if (g.kw > kTapsMax) return 1;
  int64_t P = cdiv(1024, g.cgroups);
  const int64_t ntile = g.B * g.tgroups;
  if (P > ntile) P = ntile;
  if (P > 256) P = 256;
  return static_cast<int>(P);
}

aqt_status launch_corr(bool rev, const float *xin, const float *xmul, const float *w, const float *bias,
                       const float *na, const float *nb, int swish, const ConvGeom &g, float *out, float *dfac,
                       uint32_t *absmax, hipStream_t st, bool absmax_is_zero = false) {
  const int pl = rev ? g.kw - 1 - g.pad_left : g.pad_left;
  if (absmax && !absmax_is_zero) zero_absmax_kernel<<<1, 64, 0, st>>>(absmax);
  const int64_t blocks = static_cast<int64_t>(g.cgroups) * g.tgroups * g.B;
  if (g.kw <= kTapsMax && blocks < (int64_t(1) << 31)) {
    const size_t lds = static_cast<size_t>(kTile + 2 * g.kw - 1) * 64 * sizeof(float);
    dwconv_kernel<<<static_cast<unsigned>(blocks), kThreads, lds, st>>>(xin, xmul, w, bias, na, nb, swish, rev ? 1 : 0, g,
                                                                        pl, out, dfac, absmax);
  } else {
    int64_t grid = cdiv(g.B * g.T * g.C, kThreads);
    if (grid > 8192) grid = 8192;
    dwconv_any_kernel<<<static_cast<unsigned>(grid), kThreads, 0, st>>>(xin, xmul, w, bias, na, nb, swish, rev ? 1 : 0, g,
                                                                      pl, out, dfac, absmax);
  }
  AQT_HIP(hipGetLastError());
  return AQT_OK;
}

}  // namespace

// Shape-only bound (the partial count never exceeds what an unlimited number of tiles gives).
size_t dwconv_bwd_ws_bytes(int64_t C, int kw) {
  ConvGeom g = geom(int64_t(1) << 20, kTile, C, kw, 0);
  return align_up(static_cast<size_t>(dw_partials(g)) * (kw + 1) * C * sizeof(float), 256);
}

aqt_status launch_dwconv_fwd(const float *x, const float *w, const float *bias, const float *na, const float *nb,
                             int swish, int64_t B, int64_t T, int64_t C, int kw, int pad_left, float *out, float *dfac,
                             uint32_t *absmax, hipStream_t st, bool absmax_is_zero) {
  return launch_corr(false, x, nullptr, w, bias, na, nb, swish, geom(B, T, C, kw, pad_left), out, dfac, absmax, st,
                     absmax_is_zero);
}

aqt_status launch_dwconv_bwd(const float *dout, const float *dmul, const float *x, const float *w, int64_t B, int64_t T,
                             int64_t C, int kw, int pad_left, float *dx, float *dw, float *dbias, void *ws,
                             hipStream_t st) {
  const ConvGeom g = geom(B, T, C, kw, pad_left);
  if (dx) AQT_TRY(launch_corr(true, dout, dmul, w, nullptr, nullptr, nullptr, 0, g, dx, nullptr, nullptr, st));
  if (dw || dbias) {
    float *part = static_cast<float *>(ws);
    const int P = dw_partials(g);
    if (kw <= kTapsMax) {
      const int kwp = (kw + 3) & ~3;
      const size_t lds = static_cast<size_t>(2 * kTile + 2 * kwp + 6) * 64 * sizeof(float);
      dwconv_dw_kernel<<<static_cast<unsigned>(g.cgroups) * P, kThreads, lds, st>>>(dout, dmul, x, g, P, part);
    } else {
      dwconv_dw_any_kernel<<<static_cast<unsigned>(cdiv(static_cast<int64_t>(kw + 1) * C, kThreads)), kThreads, 0, st>>>(
          dout, dmul, x, g, part);
    }
    AQT_HIP(hipGetLastError());
    dwconv_dw_fold_kernel<<<static_cast<unsigned>(cdiv(static_cast<int64_t>(kw + 1) * C, kThreads)), kThreads, 0, st>>>(
        part, P, kw, C, dw, dbias);
    AQT_HIP(hipGetLastError());
  }
  return AQT_OK;
}

}  // namespace aqt
