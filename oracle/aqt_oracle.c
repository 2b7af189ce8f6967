/*
 * CPU oracle for native quantization-aware training's quantized dense layer
 * (arxiv 2203.15952).  TEST INFRASTRUCTURE ONLY: it is the slow, plain
 * statement of what the method computes, used to check the HIP library and to
 * serve as the timed CPU baseline.  It shares no code with the HIP library and
 * the product path never calls it.
 *
 * What each function follows:
 *   oracle_quantize*      Fig. 2 (abs-max -> scale -> divide_no_nan -> +0.5 ->
 *                         floor -> cast) and Sec. 2.2 (divide the maximum by 127
 *                         for int8, by 7 for int4; channel-wise via the reduced
 *                         axis; no zero point).
 *   oracle_pack_int4      int4 storage implied by the model sizes of Table 1
 *                         (half a byte per quantized parameter); the nibble
 *                         order is this build's choice.
 *   oracle_dense_fwd*     Sec. 1 and Sec. 2.2: quantize both operands, multiply
 *                         as integers, de-quantize by multiplying with the
 *                         scales.
 *   oracle_dense_fwd_wonly*  Sec. 4.1, configurations I8W / I4W: integer weights
 *                         de-quantized to float32, float32 activations.
 *   oracle_dense_bwd      Fig. 2's stop_gradient on the scale; the rounding is
 *                         passed straight through (the paper does not state it,
 *                         straight-through is the standard reading of QAT).
 *   oracle_epilogue_dact, oracle_dense_bwd_epi
 *                         the same backward through the layer's activation
 *                         (Swish of the feed-forward module, GLU of the
 *                         convolution module, Sec. 3.2's Conformer blocks): the
 *                         chain rule with the textbook derivatives.
 *   oracle_layernorm      the normalisation in front of the feed-forward module
 *                         (Sec. 3.2's Conformer; per token over the model width,
 *                         biased variance), float64; not part of the paper's
 *                         method, glue of the chained block.
 *   oracle_depthwise_conv*, oracle_affine_swish
 *                         the float layers between the two pointwise convolutions
 *                         of the convolution module (Sec. 3.2: depthwise kernel 32;
 *                         Sec. 3.3: causal kernel 15, convolution kernels stay
 *                         float): the plain definitions and their adjoints, float64;
 *                         glue of the chained block.
 *   oracle_attention      scaled dot-product attention with softmax over a window of
 *                         frames, the float core of the self-attention module
 *                         (Sec. 3.2: heads; Sec. 3.3: left / right context): the
 *                         textbook definition in float64; glue of the chained block.
 *   oracle_attention_bwd, oracle_layernorm_bwd
 *                         the chain rule through those two, written out, float64.
 *   oracle_fake_matmul_f32  Sec. 1 / Sec. 2.2: "fake" quantization carries the integer
 *                         codes in float32 and multiplies them with float
 *                         operations; sums that need more than 24 bits are rounded.
 *
 * Arithmetic: the quantizer is binary32, one rounding per operation, because
 * the paper's listing is float32 TensorFlow and the codes depend on it.  The
 * contraction accumulates in int64 (and reports whether it would have fitted
 * int32).  De-quantization, epilogues and gradients are evaluated in binary64.
 * Build with -O2 -ffp-contract=off and without -ffast-math.
 *
 * Parity pins: every function here is pinned by tests that do not call it to
 * produce their expected values (tie table, range, half-step error bound,
 * integer-valued special case against an int64 library matmul, power-of-two
 * equivariance, an independent binary32-emulating brute force, the method's
 * error bound against the float product, gradients against a library float64
 * matmul of the de-quantized operands, hand-packed bytes; the weight-only forward
 * by a hand-worked example, one-hot activations, agreement with the integer path
 * on activations that are exact multiples of a power-of-two scale, and the
 * half-step bound against the float product; the activation derivatives by
 * closed-form values and central differences of the activation alone, the
 * backward through the activation by central differences of the de-quantized
 * layer in float64 numpy; the normalisation by a hand-worked row, zero mean and
 * unit variance of its rows, and numpy; the float32-emulated product by equality
 * with the integer product while sums fit 24 bits and a hand-worked sum that does
 * not; the depthwise convolution by its impulse response, a hand-worked causal
 * example, numpy's correlate per channel, the adjoint identity and central
 * differences for its gradients; the affine + Swish by closed-form values and
 * central differences; the attention by zero queries (window means), a one-hot
 * alignment, constant values, the zero-width window and scipy's softmax; the
 * backward of attention and normalisation by central differences of their
 * forward functions, by the zero-width window and by the orthogonality of a
 * normalised row's gradient to the constant and to the row itself).  The paper prints
 * no worked numeric example, so no pin comes from printed values.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_AXIS_ALL (-1)
#define ORACLE_EPI_NONE 0
#define ORACLE_EPI_SWISH 1
#define ORACLE_EPI_GLU 2

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

static int qmax_of(int bits) { return (1 << (bits - 1)) - 1; }

/* One element of Fig. 2 given its group's scale.  Returns the code; *pass is 1
 * when the rounded value needed no saturation and the scale is non-zero. */
static int8_t quantize_one(float x, float s, int qmax, uint8_t *pass) {
  float t = (s == 0.0f) ? 0.0f : x / s; /* divide_no_nan */
  float u = t + 0.5f;
  float r = floorf(u);
  int in_range = (r >= (float)(-qmax)) && (r <= (float)qmax);
  float c = r;
  if (c > (float)qmax) c = (float)qmax;
  if (c < (float)(-qmax)) c = (float)(-qmax);
  if (pass) *pass = (uint8_t)(in_range && (s != 0.0f));
  return (int8_t)c;
}

/* Scale of one reduction group: maximum magnitude divided by qmax (Sec. 2.2). */
static float scale_of(float m, int qmax) { return m / (float)qmax; }

/*
 * Fig. 2 with the bit-width rule of Sec. 2.2.  x is [rows, cols] row-major.
 * axis names the REDUCED axes: ORACLE_AXIS_ALL -> one scale; 0 -> reduce over
 * rows, one scale per column; 1 -> reduce over columns, one scale per row.
 * q: [rows, cols] codes.  scale: 1, cols or rows floats.  mask: nullable,
 * one byte per element (1 = gradient passes).
 * Returns 0, or 1 if a group's maximum is not finite (outputs then unspecified).
 */
int oracle_quantize(const float *x, int64_t rows, int64_t cols, int bits, int axis,
                    int8_t *q, float *scale, uint8_t *mask) {
  const int qmax = qmax_of(bits);
  int bad = 0;
  if (axis == ORACLE_AXIS_ALL) {
    float m = 0.0f;
    for (int64_t i = 0; i < rows * cols; ++i) {
      float a = fabsf(x[i]);
      if (!isfinite(a)) return 1;
      if (a > m) m = a;
    }
    float s = scale_of(m, qmax);
    scale[0] = s;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows * cols; ++i)
      q[i] = quantize_one(x[i], s, qmax, mask ? &mask[i] : NULL);
  } else if (axis == 0) {
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t c = 0; c < cols; ++c) {
      float m = 0.0f;
      int nonfinite = 0;
      for (int64_t r = 0; r < rows; ++r) {
        float a = fabsf(x[r * cols + c]);
        if (!isfinite(a)) nonfinite = 1;
        if (a > m) m = a;
      }
      if (nonfinite) { bad |= 1; continue; }
      float s = scale_of(m, qmax);
      scale[c] = s;
      for (int64_t r = 0; r < rows; ++r)
        q[r * cols + c] = quantize_one(x[r * cols + c], s, qmax, mask ? &mask[r * cols + c] : NULL);
    }
  } else if (axis == 1) {
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t r = 0; r < rows; ++r) {
      float m = 0.0f;
      int nonfinite = 0;
      for (int64_t c = 0; c < cols; ++c) {
        float a = fabsf(x[r * cols + c]);
        if (!isfinite(a)) nonfinite = 1;
        if (a > m) m = a;
      }
      if (nonfinite) { bad |= 1; continue; }
      float s = scale_of(m, qmax);
      scale[r] = s;
      for (int64_t c = 0; c < cols; ++c)
        q[r * cols + c] = quantize_one(x[r * cols + c], s, qmax, mask ? &mask[r * cols + c] : NULL);
    }
  } else {
    return 2;
  }
  return bad;
}

/*
 * The element-wise half of Fig. 2 with scales supplied by the caller instead of
 * derived from the data.  Only this form can saturate, so it is what exercises
 * a clip mask that is not all ones.  Same layout and axis meaning as above.
 */
int oracle_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int bits, int axis,
                               const float *scale, int8_t *q, uint8_t *mask) {
  const int qmax = qmax_of(bits);
  if (axis != ORACLE_AXIS_ALL && axis != 0 && axis != 1) return 2;
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) {
      float s = (axis == ORACLE_AXIS_ALL) ? scale[0] : (axis == 0 ? scale[c] : scale[r]);
      int64_t i = r * cols + c;
      q[i] = quantize_one(x[i], s, qmax, mask ? &mask[i] : NULL);
    }
  return 0;
}

/*
 * int4 storage: codes [K, N] (K = fan-in) -> bytes [N][ceil(K/2)], fan-in
 * contiguous.  Byte j of channel n holds k = 2j in its low nibble and k = 2j+1
 * in its high nibble, both two's complement; an odd K leaves the last high
 * nibble zero.
 */
void oracle_pack_int4(const int8_t *codes_kn, int64_t K, int64_t N, uint8_t *bytes) {
  const int64_t kb = (K + 1) / 2;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t j = 0; j < kb; ++j) {
      uint8_t lo = (uint8_t)codes_kn[(2 * j) * N + n] & 0xF;
      uint8_t hi = (2 * j + 1 < K) ? ((uint8_t)codes_kn[(2 * j + 1) * N + n] & 0xF) : 0;
      bytes[n * kb + j] = (uint8_t)(lo | (hi << 4));
    }
}

static double sigmoid64(double v) { return 1.0 / (1.0 + exp(-v)); }

/*
 * Integer contraction and de-quantization on already-quantized operands
 * (Sec. 2.2: de-quantize by multiplying with the scales).
 * xq [M,K] codes, s_x scalar, wq_kn [K,N] codes, s_w [N], bias nullable [N].
 * acc (nullable) [M,N] receives the integer sums as int32; y is [M,N] doubles,
 * or [M,N/2] for GLU (first half of the channels is the value, second half the
 * gate).  pre (nullable) [M,N] receives the de-quantized value before the
 * activation.  Returns 0, or 3 if any integer sum does not fit int32.
 */
int oracle_dense_fwd_q(const int8_t *xq, float s_x, const int8_t *wq_kn, const float *s_w,
                       int64_t M, int64_t K, int64_t N, const float *bias, int epilogue,
                       int32_t *acc, double *y, double *pre) {
  int overflow = 0;
  if (epilogue == ORACLE_EPI_GLU && (N % 2)) return 2;
#pragma omp parallel for schedule(static) reduction(| : overflow)
  for (int64_t m = 0; m < M; ++m) {
    double *v = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t n = 0; n < N; ++n) {
      int64_t a = 0;
      for (int64_t k = 0; k < K; ++k) a += (int64_t)xq[m * K + k] * (int64_t)wq_kn[k * N + n];
      if (a > INT32_MAX || a < INT32_MIN) overflow |= 1;
      if (acc) acc[m * N + n] = (int32_t)a;
      double d = (double)a * (double)s_x * (double)s_w[n];
      if (bias) d += (double)bias[n];
      v[n] = d;
      if (pre) pre[m * N + n] = d;
    }
    if (epilogue == ORACLE_EPI_NONE) {
      for (int64_t n = 0; n < N; ++n) y[m * N + n] = v[n];
    } else if (epilogue == ORACLE_EPI_SWISH) {
      for (int64_t n = 0; n < N; ++n) y[m * N + n] = v[n] * sigmoid64(v[n]);
    } else {
      const int64_t h = N / 2;
      for (int64_t j = 0; j < h; ++j) y[m * h + j] = v[j] * sigmoid64(v[j + h]);
    }
    free(v);
  }
  return overflow ? 3 : 0;
}

/*
 * Weight-only modes (Sec. 4.1, configurations I8W / I4W: integer weights, float32
 * activations; the weights are converted back to float for the product).
 * x [M,K] float32, wq_kn [K,N] codes, s_w [N], bias nullable [N].
 * The de-quantized weight is the float32 number w^[k,n] = s_w[n] * (float)wq[k,n]
 * (one float32 rounding, as a float32 graph would hold it); the product with x is
 * then evaluated in double, so what is returned is the exact value a float32
 * matmul of x and w^ approximates.  y [M,N] doubles ([M,N/2] for GLU), pre
 * (nullable) [M,N] the value before the activation, mag (nullable) [M,N] the sum of
 * the magnitudes of the terms, the yardstick for a float contraction.
 */
int oracle_dense_fwd_wonly(const float *x, const int8_t *wq_kn, const float *s_w,
                           int64_t M, int64_t K, int64_t N, const float *bias, int epilogue,
                           double *y, double *pre, double *mag) {
  if (epilogue == ORACLE_EPI_GLU && (N % 2)) return 2;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    double *v = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0, sa = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        const float wdq = s_w[n] * (float)wq_kn[k * N + n];   /* one binary32 rounding */
        double t = (double)x[m * K + k] * (double)wdq;
        s += t;
        sa += fabs(t);
      }
      if (bias) s += (double)bias[n];
      v[n] = s;
      if (pre) pre[m * N + n] = s;
      if (mag) mag[m * N + n] = sa + (bias ? fabs((double)bias[n]) : 0.0);
    }
    if (epilogue == ORACLE_EPI_NONE) {
      for (int64_t n = 0; n < N; ++n) y[m * N + n] = v[n];
    } else if (epilogue == ORACLE_EPI_SWISH) {
      for (int64_t n = 0; n < N; ++n) y[m * N + n] = v[n] * sigmoid64(v[n]);
    } else {
      const int64_t h = N / 2;
      for (int64_t j = 0; j < h; ++j) y[m * h + j] = v[j] * sigmoid64(v[j + h]);
    }
    free(v);
  }
  return 0;
}

void oracle_dense_fwd_wonly_sampled(const float *x, const int8_t *wq_kn, const float *s_w,
                                    int64_t K, int64_t N, const float *bias,
                                    const int64_t *idx_m, const int64_t *idx_n, int64_t count,
                                    double *pre, double *mag) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = idx_m[i], n = idx_n[i];
    double s = 0.0, sa = 0.0;
    for (int64_t k = 0; k < K; ++k) {
      const float wdq = s_w[n] * (float)wq_kn[k * N + n];
      double t = (double)x[m * K + k] * (double)wdq;
      s += t;
      sa += fabs(t);
    }
    if (bias) s += (double)bias[n];
    pre[i] = s;
    mag[i] = sa + (bias ? fabs((double)bias[n]) : 0.0);
  }
}

/*
 * The whole forward layer: quantize x per tensor and w per output channel,
 * contract as integers, de-quantize.  x [M,K], w [K,N] (fan-in major).
 * Outputs xq [M,K], s_x[1], wq_kn [K,N], s_w [N] are caller buffers; the rest
 * as oracle_dense_fwd_q.
 */
int oracle_dense_fwd(const float *x, const float *w, int64_t M, int64_t K, int64_t N,
                     int bits_x, int bits_w, const float *bias, int epilogue,
                     int8_t *xq, float *s_x, int8_t *wq_kn, float *s_w,
                     int32_t *acc, double *y, double *pre) {
  int rc = oracle_quantize(x, M, K, bits_x, ORACLE_AXIS_ALL, xq, s_x, NULL);
  if (rc) return rc;
  rc = oracle_quantize(w, K, N, bits_w, 0, wq_kn, s_w, NULL);
  if (rc) return rc;
  return oracle_dense_fwd_q(xq, s_x[0], wq_kn, s_w, M, K, N, bias, epilogue, acc, y, pre);
}

/*
 * Straight-through backward of y = (s_x xq)(s_w wq) (+ bias), scales held
 * constant (Fig. 2, stop_gradient):
 *   dx[m,k] = mask_x[m,k] * sum_n dy[m,n] * s_w[n] * wq[k,n]
 *   dw[k,n] = mask_w[k,n] * s_x * sum_m xq[m,k] * dy[m,n]
 *   dbias[n] = sum_m dy[m,n]
 * mask_x / mask_w: nullable byte masks.  A NULL mask stands for the mask abs-max
 * scaling produces: 1 wherever the group's scale is non-zero, 0 where it is zero
 * (Fig. 2's divide_no_nan passes no gradient through a zero scale; with a
 * non-zero scale the rounded value never leaves [-qmax, qmax], so nothing else
 * is ever masked).  Any of dx, dw, dbias may be NULL.  dx_abs / dw_abs (nullable) receive the sum of the magnitudes
 * of the terms, the yardstick a condition-aware comparison needs.
 */
static void dense_bwd_core(const double *dy, const int8_t *xq, float s_x, const uint8_t *mask_x,
                           const int8_t *wq_kn, const float *s_w, const uint8_t *mask_w,
                           int64_t M, int64_t K, int64_t N,
                           double *dx, double *dw, double *dbias, double *dx_abs, double *dw_abs) {
  if (dx) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
      for (int64_t k = 0; k < K; ++k) {
        double s = 0.0, sa = 0.0;
        for (int64_t n = 0; n < N; ++n) {
          double t = dy[m * N + n] * (double)s_w[n] * (double)wq_kn[k * N + n];
          s += t;
          sa += fabs(t);
        }
        double g = mask_x ? (mask_x[m * K + k] ? 1.0 : 0.0) : (s_x != 0.0f ? 1.0 : 0.0);
        dx[m * K + k] = g * s;
        if (dx_abs) dx_abs[m * K + k] = sa;
      }
  }
  if (dw) {
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < K; ++k)
      for (int64_t n = 0; n < N; ++n) {
        double s = 0.0, sa = 0.0;
        for (int64_t m = 0; m < M; ++m) {
          double t = (double)xq[m * K + k] * dy[m * N + n];
          s += t;
          sa += fabs(t);
        }
        double g = mask_w ? (mask_w[k * N + n] ? 1.0 : 0.0) : (s_w[n] != 0.0f ? 1.0 : 0.0);
        dw[k * N + n] = g * (double)s_x * s;
        if (dw_abs) dw_abs[k * N + n] = fabs((double)s_x) * sa;
      }
  }
  if (dbias) {
    for (int64_t n = 0; n < N; ++n) {
      double s = 0.0;
      for (int64_t m = 0; m < M; ++m) s += dy[m * N + n];
      dbias[n] = s;
    }
  }
}

void oracle_dense_bwd(const float *dy, const int8_t *xq, float s_x, const uint8_t *mask_x,
                      const int8_t *wq_kn, const float *s_w, const uint8_t *mask_w,
                      int64_t M, int64_t K, int64_t N,
                      double *dx, double *dw, double *dbias, double *dx_abs, double *dw_abs) {
  double *d = (double *)malloc((size_t)M * (size_t)N * sizeof(double));
  for (int64_t i = 0; i < M * N; ++i) d[i] = (double)dy[i];
  dense_bwd_core(d, xq, s_x, mask_x, wq_kn, s_w, mask_w, M, K, N, dx, dw, dbias, dx_abs, dw_abs);
  free(d);
}

/*
 * Derivative factors of the layer's activation with respect to the value v it is
 * applied to (v = de-quantized product + bias), float64:
 *   none : dact[m,n] = 1
 *   Swish: out = v s(v), s the logistic function:  dact = s(v) (1 + v (1 - s(v)))
 *   GLU  : out[m,j] = a s(g), a = v[m,j], g = v[m,j+N/2]:
 *          dact[m,j] = s(g)   (d out / d a),   dact[m,j+N/2] = a s(g) (1 - s(g))   (d out / d g)
 * so that d v[m,n] = d out[m, n mod out_cols] * dact[m,n] in every case.
 * pre and dact are [M,N].
 */
int oracle_epilogue_dact(const double *pre, int64_t M, int64_t N, int epilogue, double *dact) {
  if (epilogue == ORACLE_EPI_GLU && (N % 2)) return 2;
  const int64_t h = N / 2;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double v = pre[m * N + n], d;
      if (epilogue == ORACLE_EPI_NONE) {
        d = 1.0;
      } else if (epilogue == ORACLE_EPI_SWISH) {
        double sg = sigmoid64(v);
        d = sg * (1.0 + v * (1.0 - sg));
      } else if (n < h) {
        d = sigmoid64(pre[m * N + n + h]);
      } else {
        double sg = sigmoid64(v);
        d = pre[m * N + n - h] * sg * (1.0 - sg);
      }
      dact[m * N + n] = d;
    }
  return 0;
}

/*
 * Straight-through backward through the activation: dout is the gradient with
 * respect to the layer's output ([M,N], or [M,N/2] for GLU), pre [M,N] the value
 * the activation was applied to.  The gradient with respect to that value,
 * dv = dout * dact (chain rule), then takes the place of dy in oracle_dense_bwd.
 * dv_out (nullable) [M,N] receives it.
 */
int oracle_dense_bwd_epi(const float *dout, const double *pre, int epilogue,
                         const int8_t *xq, float s_x, const uint8_t *mask_x,
                         const int8_t *wq_kn, const float *s_w, const uint8_t *mask_w,
                         int64_t M, int64_t K, int64_t N,
                         double *dx, double *dw, double *dbias, double *dx_abs, double *dw_abs,
                         double *dv_out) {
  double *dact = (double *)malloc((size_t)M * (size_t)N * sizeof(double));
  int rc = oracle_epilogue_dact(pre, M, N, epilogue, dact);
  if (rc) { free(dact); return rc; }
  const int64_t oc = (epilogue == ORACLE_EPI_GLU) ? N / 2 : N;
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) dact[m * N + n] *= (double)dout[m * oc + (n % oc)];
  if (dv_out) memcpy(dv_out, dact, (size_t)M * (size_t)N * sizeof(double));
  dense_bwd_core(dact, xq, s_x, mask_x, wq_kn, s_w, mask_w, M, K, N, dx, dw, dbias, dx_abs, dw_abs);
  free(dact);
  return 0;
}

/*
 * Layer normalisation of each row of x [M,D] over its D entries, float64:
 * mean and biased variance of the row, y = (x - mean) / sqrt(var + eps) * gamma + beta;
 * gamma / beta nullable (1 / 0).
 */
void oracle_layernorm(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                      double eps, double *y) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    double mean = 0.0, var = 0.0;
    for (int64_t d = 0; d < D; ++d) mean += (double)x[m * D + d];
    mean /= (double)D;
    for (int64_t d = 0; d < D; ++d) {
      double c = (double)x[m * D + d] - mean;
      var += c * c;
    }
    var /= (double)D;
    const double r = 1.0 / sqrt(var + eps);
    for (int64_t d = 0; d < D; ++d) {
      double v = ((double)x[m * D + d] - mean) * r;
      if (gamma) v *= (double)gamma[d];
      if (beta) v += (double)beta[d];
      y[m * D + d] = v;
    }
  }
}

/*
 * "Fake" quantization's product (Sec. 1, Sec. 2.2): the integer codes are carried
 * as float32 numbers and multiplied and added with float32 operations, one
 * rounding per operation, summed in order of k.  Equal to the integer product
 * as long as every partial sum fits the 24-bit significand; beyond that the
 * sums are rounded.  out [M,N] float32.
 */
void oracle_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N,
                            float *out) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      float a = 0.0f;
      for (int64_t k = 0; k < K; ++k) {
        float p = (float)xq[m * K + k] * (float)wq_kn[k * N + n];   /* exact: |p| <= 127 * 127 */
        a = a + p;                                                 /* one binary32 rounding */
      }
      out[m * N + n] = a;
    }
}

/*
 * Depthwise convolution along time, the float layer between the two pointwise
 * convolutions of the Conformer convolution module (Sec. 3.2: kernel size 32;
 * Sec. 3.3: causal, kernel size 15, and the convolution kernels are not
 * quantized).  x [B,T,C]: B utterances of T frames, C channels; w [kw,C]; bias
 * nullable [C].  Frames outside an utterance count as zero:
 *   out[b,t,c] = bias[c] + sum_j w[j,c] * x[b, t + j - pad_left, c],  0 <= j < kw.
 * pad_left = kw - 1 makes the layer causal.  float64; out_abs (nullable) gets the
 * sum of the absolute values of the same terms.
 */
void oracle_depthwise_conv(const float *x, const float *w, const float *bias, int64_t B, int64_t T,
                           int64_t C, int64_t kw, int64_t pad_left, double *out, double *out_abs) {
#pragma omp parallel for schedule(static)
  for (int64_t bt = 0; bt < B * T; ++bt) {
    const int64_t b = bt / T, t = bt % T;
    for (int64_t c = 0; c < C; ++c) {
      double a = bias ? (double)bias[c] : 0.0, ab = fabs(a);
      for (int64_t j = 0; j < kw; ++j) {
        const int64_t u = t + j - pad_left;
        if (u < 0 || u >= T) continue;
        const double p = (double)w[j * C + c] * (double)x[(b * T + u) * C + c];
        a += p;
        ab += fabs(p);
      }
      out[bt * C + c] = a;
      if (out_abs) out_abs[bt * C + c] = ab;
    }
  }
}

/*
 * Gradients of oracle_depthwise_conv for an upstream gradient dout [B,T,C] (float64):
 *   dx[b,u,c]  = sum_j w[j,c] * dout[b, u - j + pad_left, c]
 *   dw[j,c]    = sum_{b,t} dout[b,t,c] * x[b, t + j - pad_left, c]
 *   dbias[c]   = sum_{b,t} dout[b,t,c]
 * each nullable; dx_abs / dw_abs (nullable) get the sums of absolute terms.
 */
void oracle_depthwise_conv_bwd(const double *dout, const float *x, const float *w, int64_t B, int64_t T,
                               int64_t C, int64_t kw, int64_t pad_left, double *dx, double *dw,
                               double *dbias, double *dx_abs, double *dw_abs) {
  if (dx) {
#pragma omp parallel for schedule(static)
    for (int64_t bu = 0; bu < B * T; ++bu) {
      const int64_t b = bu / T, u = bu % T;
      for (int64_t c = 0; c < C; ++c) {
        double a = 0.0, ab = 0.0;
        for (int64_t j = 0; j < kw; ++j) {
          const int64_t t = u - j + pad_left;
          if (t < 0 || t >= T) continue;
          const double p = (double)w[j * C + c] * dout[(b * T + t) * C + c];
          a += p;
          ab += fabs(p);
        }
        dx[bu * C + c] = a;
        if (dx_abs) dx_abs[bu * C + c] = ab;
      }
    }
  }
  if (dw) {
#pragma omp parallel for schedule(static)
    for (int64_t jc = 0; jc < kw * C; ++jc) {
      const int64_t j = jc / C, c = jc % C;
      double a = 0.0, ab = 0.0;
      for (int64_t b = 0; b < B; ++b)
        for (int64_t t = 0; t < T; ++t) {
          const int64_t u = t + j - pad_left;
          if (u < 0 || u >= T) continue;
          const double p = dout[(b * T + t) * C + c] * (double)x[(b * T + u) * C + c];
          a += p;
          ab += fabs(p);
        }
      dw[jc] = a;
      if (dw_abs) dw_abs[jc] = ab;
    }
  }
  if (dbias) {
    for (int64_t c = 0; c < C; ++c) {
      double a = 0.0;
      for (int64_t bt = 0; bt < B * T; ++bt) a += dout[bt * C + c];
      dbias[c] = a;
    }
  }
}

/*
 * The normalisation after the depthwise convolution in the form it takes once its
 * statistics are fixed (one scale a[c] and one shift b[c] per channel, both nullable:
 * 1 and 0), followed by Swish (Sec. 3.2's convolution module):
 *   n = v * a[c] + b[c];  out = n * sigmoid(n);  dfac = d out / d v = a[c] * swish'(n)
 * with swish'(n) = s (1 + n (1 - s)), s = sigmoid(n).  float64; out, dfac nullable.
 */
void oracle_affine_swish(const double *v, int64_t M, int64_t C, const float *a, const float *b,
                         double *out, double *dfac) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t c = 0; c < C; ++c) {
      const double ac = a ? (double)a[c] : 1.0;
      const double n = v[m * C + c] * ac + (b ? (double)b[c] : 0.0);
      const double s = sigmoid64(n);
      if (out) out[m * C + c] = n * s;
      if (dfac) dfac[m * C + c] = ac * s * (1.0 + n * (1.0 - s));
    }
}

/*
 * Scaled dot-product self-attention over each utterance, the float core between the
 * quantized projections of the Conformer's self-attention module (Sec. 3.2: 4 or 8 heads;
 * Sec. 3.3: a limited left context and, in the non-causal encoder, a limited right context).
 * qkv [B,T,3D] holds queries, keys and values in three column blocks of width D, head h in
 * columns h*dh .. (h+1)*dh of each block, dh = D / heads.  For query frame t of utterance b
 * and head h, over the key frames j of the same utterance with t - left <= j <= t + right
 * (left / right < 0: no limit on that side):
 *   s_j = (q_t . k_j) / sqrt(dh);  p = softmax_j(s);  ctx[b,t,h*dh + d] = sum_j p_j v_j[d]
 * float64.  smag [B,T,heads] (nullable): the largest sum_d |q_d k_jd| / sqrt(dh) over the window;
 * vmag [B,T,D] (nullable): sum_j p_j |v_j[d]|; both only feed error bounds.
 */
int oracle_attention(const float *qkv, int64_t B, int64_t T, int64_t D, int64_t heads, int64_t left,
                     int64_t right, double *ctx, double *smag, double *vmag) {
  if (heads < 1 || D % heads) return 2;
  const int64_t dh = D / heads;
  const double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for schedule(static)
  for (int64_t bt = 0; bt < B * T; ++bt) {
    const int64_t b = bt / T, t = bt % T;
    const int64_t j0 = (left < 0 || t - left < 0) ? 0 : t - left;
    const int64_t j1 = (right < 0 || t + right > T - 1) ? T - 1 : t + right;
    double *s = (double *)malloc((size_t)(j1 - j0 + 1) * sizeof(double));
    for (int64_t h = 0; h < heads; ++h) {
      const float *q = qkv + bt * 3 * D + h * dh;
      double mx = -INFINITY, mg = 0.0;
      for (int64_t j = j0; j <= j1; ++j) {
        const float *k = qkv + (b * T + j) * 3 * D + D + h * dh;
        double a = 0.0, ab = 0.0;
        for (int64_t d = 0; d < dh; ++d) {
          a += (double)q[d] * (double)k[d];
          ab += fabs((double)q[d] * (double)k[d]);
        }
        s[j - j0] = a * scale;
        if (s[j - j0] > mx) mx = s[j - j0];
        if (ab * scale > mg) mg = ab * scale;
      }
      double sum = 0.0;
      for (int64_t j = j0; j <= j1; ++j) {
        s[j - j0] = exp(s[j - j0] - mx);
        sum += s[j - j0];
      }
      for (int64_t d = 0; d < dh; ++d) {
        double a = 0.0, ab = 0.0;
        for (int64_t j = j0; j <= j1; ++j) {
          const double v = (double)qkv[(b * T + j) * 3 * D + 2 * D + h * dh + d];
          a += s[j - j0] * v;
          ab += s[j - j0] * fabs(v);
        }
        ctx[bt * D + h * dh + d] = a / sum;
        if (vmag) vmag[bt * D + h * dh + d] = ab / sum;
      }
      if (smag) smag[bt * heads + h] = mg;
    }
    free(s);
  }
  return 0;
}

/*
 * Gradients of oracle_attention for an upstream gradient dctx [B,T,D] (float64), the chain
 * rule through softmax and the two products written out:
 *   dP_tj = dctx_t . v_j;   dS_tj = p_tj (dP_tj - sum_i p_ti dP_ti);
 *   dq_t = sum_j dS_tj k_j / sqrt(dh);  dk_j = sum_t dS_tj q_t / sqrt(dh);  dv_j = sum_t p_tj dctx_t
 * dqkv [B,T,3D] in the layout of qkv.  mag (nullable, same shape): the sums of the absolute
 * values of the terms, with |dS| bounded by p (|dP| + sum_i p_i |dP_i|); only feeds error bounds.
 */
int oracle_attention_bwd(const float *qkv, const double *dctx, int64_t B, int64_t T, int64_t D, int64_t heads,
                         int64_t left, int64_t right, double *dqkv, double *mag) {
  if (heads < 1 || D % heads) return 2;
  const int64_t dh = D / heads;
  const double scale = 1.0 / sqrt((double)dh);
  memset(dqkv, 0, (size_t)(B * T * 3 * D) * sizeof(double));
  if (mag) memset(mag, 0, (size_t)(B * T * 3 * D) * sizeof(double));
#pragma omp parallel for schedule(dynamic)
  for (int64_t bh = 0; bh < B * heads; ++bh) {
    const int64_t b = bh / heads, h = bh % heads;
    double *p = (double *)malloc((size_t)T * sizeof(double));
    double *dp = (double *)malloc((size_t)T * sizeof(double));
    for (int64_t t = 0; t < T; ++t) {
      const int64_t j0 = (left < 0 || t - left < 0) ? 0 : t - left;
      const int64_t j1 = (right < 0 || t + right > T - 1) ? T - 1 : t + right;
      const float *q = qkv + (b * T + t) * 3 * D + h * dh;
      const double *g = dctx + (b * T + t) * D + h * dh;
      double mx = -INFINITY, sum = 0.0, dd = 0.0, dda = 0.0;
      for (int64_t j = j0; j <= j1; ++j) {
        const float *k = qkv + (b * T + j) * 3 * D + D + h * dh;
        double a = 0.0;
        for (int64_t d = 0; d < dh; ++d) a += (double)q[d] * (double)k[d];
        p[j] = a * scale;
        if (p[j] > mx) mx = p[j];
      }
      for (int64_t j = j0; j <= j1; ++j) {
        p[j] = exp(p[j] - mx);
        sum += p[j];
      }
      for (int64_t j = j0; j <= j1; ++j) {
        const float *v = qkv + (b * T + j) * 3 * D + 2 * D + h * dh;
        double a = 0.0;
        for (int64_t d = 0; d < dh; ++d) a += g[d] * (double)v[d];
        p[j] /= sum;
        dp[j] = a;
        dd += p[j] * a;
        dda += p[j] * fabs(a);
      }
      for (int64_t j = j0; j <= j1; ++j) {
        const double ds = p[j] * (dp[j] - dd) * scale, dsa = p[j] * (fabs(dp[j]) + dda) * scale;
        const int64_t qo = (b * T + t) * 3 * D + h * dh, ko = (b * T + j) * 3 * D + D + h * dh, vo = ko + D;
        for (int64_t d = 0; d < dh; ++d) {
          dqkv[qo + d] += ds * (double)qkv[ko + d];
          dqkv[ko + d] += ds * (double)qkv[qo + d];
          dqkv[vo + d] += p[j] * g[d];
          if (mag) {
            mag[qo + d] += dsa * fabs((double)qkv[ko + d]);
            mag[ko + d] += dsa * fabs((double)qkv[qo + d]);
            mag[vo + d] += p[j] * fabs(g[d]);
          }
        }
      }
    }
    free(p);
    free(dp);
  }
  return 0;
}

/*
 * Gradients of oracle_layernorm for an upstream gradient dy [M,D] (float64).  With
 * xh = (x - mean) / sqrt(var + eps) and g = dy * gamma:
 *   dx = (g - mean_row(g) - xh mean_row(g xh)) / sqrt(var + eps);  dgamma = sum_m dy xh;  dbeta = sum_m dy
 * dgamma / dbeta nullable.
 */
void oracle_layernorm_bwd(const float *x, int64_t M, int64_t D, const float *gamma, double eps, const double *dy,
                          double *dx, double *dgamma, double *dbeta) {
  if (dgamma) memset(dgamma, 0, (size_t)D * sizeof(double));
  if (dbeta) memset(dbeta, 0, (size_t)D * sizeof(double));
  for (int64_t m = 0; m < M; ++m) {
    double mean = 0.0, var = 0.0, mg = 0.0, mgx = 0.0;
    for (int64_t d = 0; d < D; ++d) mean += (double)x[m * D + d];
    mean /= (double)D;
    for (int64_t d = 0; d < D; ++d) {
      const double c = (double)x[m * D + d] - mean;
      var += c * c;
    }
    var /= (double)D;
    const double r = 1.0 / sqrt(var + eps);
    for (int64_t d = 0; d < D; ++d) {
      const double xh = ((double)x[m * D + d] - mean) * r;
      const double g = dy[m * D + d] * (gamma ? (double)gamma[d] : 1.0);
      mg += g;
      mgx += g * xh;
      if (dgamma) dgamma[d] += dy[m * D + d] * xh;
      if (dbeta) dbeta[d] += dy[m * D + d];
    }
    mg /= (double)D;
    mgx /= (double)D;
    for (int64_t d = 0; d < D; ++d) {
      const double xh = ((double)x[m * D + d] - mean) * r;
      const double g = dy[m * D + d] * (gamma ? (double)gamma[d] : 1.0);
      dx[m * D + d] = (g - mg - xh * mgx) * r;
    }
  }
}

/*
 * Sampled variants for full-size checks: the same definitions evaluated only
 * at listed output positions, so a test can afford the benchmark shapes.
 * idx_m/idx_n (or idx_m/idx_k, idx_k/idx_n) have `count` entries each.
 */
void oracle_dense_fwd_q_sampled(const int8_t *xq, float s_x, const int8_t *wq_kn, const float *s_w,
                                int64_t K, int64_t N, const float *bias,
                                const int64_t *idx_m, const int64_t *idx_n, int64_t count,
                                int64_t *acc, double *pre) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = idx_m[i], n = idx_n[i], a = 0;
    for (int64_t k = 0; k < K; ++k) a += (int64_t)xq[m * K + k] * (int64_t)wq_kn[k * N + n];
    acc[i] = a;
    double d = (double)a * (double)s_x * (double)s_w[n];
    if (bias) d += (double)bias[n];
    pre[i] = d;
  }
}

void oracle_dense_bwd_dx_sampled(const float *dy, const int8_t *wq_kn, const float *s_w,
                                 int64_t K, int64_t N, const int64_t *idx_m, const int64_t *idx_k,
                                 int64_t count, double *dx, double *dx_abs) {
  (void)K;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t m = idx_m[i], k = idx_k[i];
    double s = 0.0, sa = 0.0;
    for (int64_t n = 0; n < N; ++n) {
      double t = (double)dy[m * N + n] * (double)s_w[n] * (double)wq_kn[k * N + n];
      s += t;
      sa += fabs(t);
    }
    dx[i] = s;
    dx_abs[i] = sa;
  }
}

void oracle_dense_bwd_dw_sampled(const float *dy, const int8_t *xq, float s_x,
                                 int64_t M, int64_t K, int64_t N, const int64_t *idx_k,
                                 const int64_t *idx_n, int64_t count, double *dw, double *dw_abs) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < count; ++i) {
    int64_t k = idx_k[i], n = idx_n[i];
    double s = 0.0, sa = 0.0;
    for (int64_t m = 0; m < M; ++m) {
      double t = (double)xq[m * K + k] * (double)dy[m * N + n];
      s += t;
      sa += fabs(t);
    }
    dw[i] = (double)s_x * s;
    dw_abs[i] = fabs((double)s_x) * sa;
  }
}
