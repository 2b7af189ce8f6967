/*
 * Host-sanitizer driver for the CPU oracle.  Built by tests/test_oracle_sanitize.py
 * together with oracle/aqt_oracle.c under -fsanitize=address,undefined and run as
 * a subprocess: every oracle routine is called on small ragged shapes with
 * buffers allocated at exactly the documented sizes, so an out-of-bounds index,
 * a misaligned access or a signed overflow anywhere in the oracle aborts the run.
 * A few values fixed by the paper are checked on the way (the rounding of Fig. 2
 * at ties; 127 and 7 as the divisors of Sec. 2.2).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_quantize(const float *x, int64_t rows, int64_t cols, int bits, int axis, int8_t *q, float *scale,
                    uint8_t *mask);
int oracle_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int bits, int axis, const float *scale,
                               int8_t *q, uint8_t *mask);
void oracle_pack_int4(const int8_t *codes_kn, int64_t K, int64_t N, uint8_t *bytes);
int oracle_dense_fwd_q(const int8_t *xq, float s_x, const int8_t *wq_kn, const float *s_w, int64_t M, int64_t K,
                       int64_t N, const float *bias, int epilogue, int32_t *acc, double *y, double *pre);
int oracle_dense_fwd_wonly(const float *x, const int8_t *wq_kn, const float *s_w, int64_t M, int64_t K, int64_t N,
                           const float *bias, int epilogue, double *y, double *pre, double *mag);
void oracle_dense_fwd_wonly_sampled(const float *x, const int8_t *wq_kn, const float *s_w, int64_t K, int64_t N,
                                    const float *bias, const int64_t *idx_m, const int64_t *idx_n, int64_t count,
                                    double *pre, double *mag);
int oracle_dense_fwd(const float *x, const float *w, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w,
                     const float *bias, int epilogue, int8_t *xq, float *s_x, int8_t *wq_kn, float *s_w,
                     int32_t *acc, double *y, double *pre);
void oracle_dense_bwd(const float *dy, const int8_t *xq, float s_x, const uint8_t *mask_x, const int8_t *wq_kn,
                      const float *s_w, const uint8_t *mask_w, int64_t M, int64_t K, int64_t N, double *dx,
                      double *dw, double *dbias, double *dx_abs, double *dw_abs);
int oracle_epilogue_dact(const double *pre, int64_t M, int64_t N, int epilogue, double *dact);
int oracle_dense_bwd_epi(const float *dout, const double *pre, int epilogue, const int8_t *xq, float s_x,
                         const uint8_t *mask_x, const int8_t *wq_kn, const float *s_w, const uint8_t *mask_w,
                         int64_t M, int64_t K, int64_t N, double *dx, double *dw, double *dbias, double *dx_abs,
                         double *dw_abs, double *dv_out);
void oracle_layernorm(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta, double eps,
                      double *y);
void oracle_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N, float *out);
void oracle_depthwise_conv(const float *x, const float *w, const float *bias, int64_t B, int64_t T, int64_t C,
                           int64_t kw, int64_t pad_left, double *out, double *out_abs);
void oracle_depthwise_conv_bwd(const double *dout, const float *x, const float *w, int64_t B, int64_t T, int64_t C,
                               int64_t kw, int64_t pad_left, double *dx, double *dw, double *dbias, double *dx_abs,
                               double *dw_abs);
int oracle_attention(const float *qkv, int64_t B, int64_t T, int64_t D, int64_t heads, int64_t left, int64_t right,
                     double *ctx, double *smag, double *vmag);
int oracle_attention_bwd(const float *qkv, const double *dctx, int64_t B, int64_t T, int64_t D, int64_t heads,
                         int64_t left, int64_t right, double *dqkv, double *mag);
void oracle_layernorm_bwd(const float *x, int64_t M, int64_t D, const float *gamma, double eps, const double *dy,
                          double *dx, double *dgamma, double *dbeta);
void oracle_affine_swish(const double *v, int64_t M, int64_t C, const float *a, const float *b, double *out,
                         double *dfac);
void oracle_dense_fwd_q_sampled(const int8_t *xq, float s_x, const int8_t *wq_kn, const float *s_w, int64_t K,
                                int64_t N, const float *bias, const int64_t *idx_m, const int64_t *idx_n,
                                int64_t count, int64_t *acc, double *pre);
void oracle_dense_bwd_dx_sampled(const float *dy, const int8_t *wq_kn, const float *s_w, int64_t K, int64_t N,
                                 const int64_t *idx_m, const int64_t *idx_k, int64_t count, double *dx,
                                 double *dx_abs);
void oracle_dense_bwd_dw_sampled(const float *dy, const int8_t *xq, float s_x, int64_t M, int64_t K, int64_t N,
                                 const int64_t *idx_k, const int64_t *idx_n, int64_t count, double *dw,
                                 double *dw_abs);

static uint32_t lcg_state = 12345u;
static float next_unit(void) { /* deterministic values in (-1, 1) */
  lcg_state = lcg_state * 1664525u + 1013904223u;
  return (float)((int32_t)(lcg_state >> 8) - (1 << 23)) / (float)(1 << 23);
}

static void *need(size_t n) {
  void *p = malloc(n ? n : 1);
  if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
  return p;
}

#define CHECK(c)                                                        \
  do {                                                                  \
    if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(2); } \
  } while (0)

static void one_shape(int64_t M, int64_t K, int64_t N, int bits_x, int bits_w) {
  float *x = need(sizeof(float) * M * K), *w = need(sizeof(float) * K * N), *dy = need(sizeof(float) * M * N);
  float *bias = need(sizeof(float) * N);
  for (int64_t i = 0; i < M * K; ++i) x[i] = 3.0f * next_unit();
  for (int64_t i = 0; i < K * N; ++i) w[i] = next_unit();
  for (int64_t i = 0; i < M * N; ++i) dy[i] = 0.1f * next_unit();
  for (int64_t i = 0; i < N; ++i) bias[i] = next_unit();
  if (N > 1) for (int64_t k = 0; k < K; ++k) w[k * N + 1] = 0.0f; /* a zero-scale channel */

  int8_t *xq = need(M * K), *wq = need(K * N);
  uint8_t *mx = need(M * K), *mw = need(K * N);
  float *s_x = need(sizeof(float)), *s_w = need(sizeof(float) * N);
  float *s_row = need(sizeof(float) * M);
  CHECK(oracle_quantize(x, M, K, bits_x, -1, xq, s_x, mx) == 0);
  CHECK(oracle_quantize(x, M, K, bits_x, 1, xq, s_row, NULL) == 0);
  CHECK(oracle_quantize(x, M, K, bits_x, -1, xq, s_x, NULL) == 0);
  CHECK(oracle_quantize(w, K, N, bits_w, 0, wq, s_w, mw) == 0);
  CHECK(oracle_quantize(w, K, N, bits_w, 7, wq, s_w, mw) == 2);
  const int qx = (1 << (bits_x - 1)) - 1, qw = (1 << (bits_w - 1)) - 1;
  for (int64_t i = 0; i < M * K; ++i) CHECK(xq[i] >= -qx && xq[i] <= qx);
  for (int64_t i = 0; i < K * N; ++i) CHECK(wq[i] >= -qw && wq[i] <= qw);
  CHECK(oracle_quantize_with_scale(w, K, N, bits_w, 0, s_w, wq, mw) == 0);

  uint8_t *packed = need((size_t)N * ((K + 1) / 2));
  oracle_pack_int4(wq, K, N, packed);

  int32_t *acc = need(sizeof(int32_t) * M * N);
  double *y = need(sizeof(double) * M * N), *pre = need(sizeof(double) * M * N), *mag = need(sizeof(double) * M * N);
  double *y_glu = need(sizeof(double) * M * (N / 2 ? N / 2 : 1));
  for (int epi = 0; epi < 2; ++epi) {
    CHECK(oracle_dense_fwd_q(xq, s_x[0], wq, s_w, M, K, N, epi ? bias : NULL, epi, acc, y, pre) == 0);
    CHECK(oracle_dense_fwd_wonly(x, wq, s_w, M, K, N, epi ? NULL : bias, epi, y, pre, mag) == 0);
  }
  if (N % 2 == 0) {
    CHECK(oracle_dense_fwd_q(xq, s_x[0], wq, s_w, M, K, N, bias, 2, NULL, y_glu, NULL) == 0);
    CHECK(oracle_dense_fwd_wonly(x, wq, s_w, M, K, N, bias, 2, y_glu, NULL, NULL) == 0);
  } else {
    CHECK(oracle_dense_fwd_q(xq, s_x[0], wq, s_w, M, K, N, bias, 2, NULL, y_glu, NULL) == 2);
  }
  CHECK(oracle_dense_fwd(x, w, M, K, N, bits_x, bits_w, bias, 1, xq, s_x, wq, s_w, acc, y, pre) == 0);

  double *dx = need(sizeof(double) * M * K), *dxa = need(sizeof(double) * M * K);
  double *dw = need(sizeof(double) * K * N), *dwa = need(sizeof(double) * K * N), *db = need(sizeof(double) * N);
  oracle_dense_bwd(dy, xq, s_x[0], mx, wq, s_w, mw, M, K, N, dx, dw, db, dxa, dwa);
  oracle_dense_bwd(dy, xq, s_x[0], NULL, wq, s_w, NULL, M, K, N, dx, dw, NULL, NULL, NULL);
  if (N > 1) for (int64_t k = 0; k < K; ++k) CHECK(dw[k * N + 1] == 0.0); /* zero scale passes no gradient */
  oracle_dense_bwd(dy, xq, s_x[0], NULL, wq, s_w, NULL, M, K, N, NULL, NULL, db, NULL, NULL);

  /* backward through the activations, the normalisation, the float32-emulated product */
  double *dv = need(sizeof(double) * M * N), *dact = need(sizeof(double) * M * N);
  CHECK(oracle_dense_fwd_q(xq, s_x[0], wq, s_w, M, K, N, bias, 0, acc, y, pre) == 0);
  for (int epi = 0; epi < 3; ++epi) {
    if (epi == 2 && (N % 2)) {
      CHECK(oracle_epilogue_dact(pre, M, N, epi, dact) == 2);
      continue;
    }
    CHECK(oracle_epilogue_dact(pre, M, N, epi, dact) == 0);
    /* dy doubles as dout: [M,N] covers [M,N/2] */
    CHECK(oracle_dense_bwd_epi(dy, pre, epi, xq, s_x[0], mx, wq, s_w, mw, M, K, N, dx, dw, db, dxa, dwa, dv) == 0);
    CHECK(oracle_dense_bwd_epi(dy, pre, epi, xq, s_x[0], NULL, wq, s_w, NULL, M, K, N, dx, NULL, NULL, NULL, NULL, NULL) == 0);
  }
  double *ln = need(sizeof(double) * M * K);
  float *gam = need(sizeof(float) * K);
  for (int64_t i = 0; i < K; ++i) gam[i] = 1.0f + 0.1f * next_unit();
  oracle_layernorm(x, M, K, NULL, NULL, 1e-6, ln);
  oracle_layernorm(x, M, K, gam, gam, 1e-6, ln);
  float *fk = need(sizeof(float) * M * N);
  oracle_fake_matmul_f32(xq, wq, M, K, N, fk);
  CHECK(oracle_dense_fwd_q(xq, s_x[0], wq, s_w, M, K, N, NULL, 0, acc, y, pre) == 0);
  for (int64_t i = 0; i < M * N; ++i) CHECK((int32_t)fk[i] == acc[i]);   /* small K: sums fit 24 bits */
  free(dv); free(dact); free(ln); free(gam); free(fk);
  oracle_dense_bwd(dy, xq, s_x[0], NULL, wq, s_w, NULL, M, K, N, dx, NULL, NULL, NULL, NULL);

  const int64_t cnt = 5;
  int64_t im[5], in[5], ik[5];
  for (int i = 0; i < 5; ++i) { im[i] = (i * 7) % M; in[i] = (i * 3) % N; ik[i] = (i * 5) % K; }
  im[4] = M - 1; in[4] = N - 1; ik[4] = K - 1;
  int64_t acc_s[5];
  double pre_s[5], mag_s[5];
  oracle_dense_fwd_q_sampled(xq, s_x[0], wq, s_w, K, N, bias, im, in, cnt, acc_s, pre_s);
  for (int i = 0; i < 5; ++i) CHECK(acc_s[i] == (int64_t)acc[im[i] * N + in[i]]);
  oracle_dense_fwd_wonly_sampled(x, wq, s_w, K, N, NULL, im, in, cnt, pre_s, mag_s);
  oracle_dense_bwd_dx_sampled(dy, wq, s_w, K, N, im, ik, cnt, pre_s, mag_s);
  for (int i = 0; i < 5; ++i) CHECK(fabs(pre_s[i] - dx[im[i] * K + ik[i]]) <= 1e-12 * (mag_s[i] + 1e-300));
  oracle_dense_bwd_dw_sampled(dy, xq, s_x[0], M, K, N, ik, in, cnt, pre_s, mag_s);

  free(x); free(w); free(dy); free(bias); free(xq); free(wq); free(mx); free(mw); free(s_x); free(s_w);
  free(s_row); free(packed); free(acc); free(y); free(pre); free(mag); free(y_glu); free(dx); free(dxa);
  free(dw); free(dwa); free(db);
}

/* depthwise convolution, its gradients and the affine + Swish on exactly sized buffers */
static void one_conv(int64_t B, int64_t T, int64_t C, int64_t kw, int64_t pad_left) {
  const size_t n = (size_t)(B * T * C);
  float *x = need(n * sizeof(float)), *w = need((size_t)(kw * C) * sizeof(float)), *b = need((size_t)C * sizeof(float));
  double *out = need(n * sizeof(double)), *ab = need(n * sizeof(double)), *dx = need(n * sizeof(double));
  double *dxa = need(n * sizeof(double)), *dw = need((size_t)(kw * C) * sizeof(double));
  double *dwa = need((size_t)(kw * C) * sizeof(double)), *db = need((size_t)C * sizeof(double));
  for (size_t i = 0; i < n; ++i) x[i] = next_unit();
  for (int64_t i = 0; i < kw * C; ++i) w[i] = next_unit();
  for (int64_t i = 0; i < C; ++i) b[i] = next_unit();
  oracle_depthwise_conv(x, w, b, B, T, C, kw, pad_left, out, ab);
  oracle_depthwise_conv(x, w, NULL, B, T, C, kw, pad_left, out, NULL);
  oracle_depthwise_conv_bwd(out, x, w, B, T, C, kw, pad_left, dx, dw, db, dxa, dwa);
  oracle_depthwise_conv_bwd(out, x, w, B, T, C, kw, pad_left, dx, NULL, NULL, NULL, NULL);
  oracle_depthwise_conv_bwd(out, x, w, B, T, C, kw, pad_left, NULL, dw, db, NULL, NULL);
  oracle_affine_swish(out, B * T, C, b, b, dx, dxa);
  oracle_affine_swish(out, B * T, C, NULL, NULL, dx, NULL);
  oracle_affine_swish(out, B * T, C, b, NULL, NULL, dxa);
  for (size_t i = 0; i < n; ++i) CHECK(isfinite(dx[i]) && isfinite(dxa[i]));
  free(x); free(w); free(b); free(out); free(ab); free(dx); free(dxa); free(dw); free(dwa); free(db);
}

/* attention on exactly sized buffers, every kind of window */
static void one_attention(int64_t B, int64_t T, int64_t D, int64_t heads) {
  const size_t n = (size_t)(B * T * D);
  float *qkv = need(3 * n * sizeof(float));
  double *ctx = need(n * sizeof(double)), *vm = need(n * sizeof(double));
  double *sm = need((size_t)(B * T * heads) * sizeof(double));
  for (size_t i = 0; i < 3 * n; ++i) qkv[i] = next_unit();
  CHECK(oracle_attention(qkv, B, T, D, heads, -1, -1, ctx, sm, vm) == 0);
  CHECK(oracle_attention(qkv, B, T, D, heads, 0, 0, ctx, NULL, NULL) == 0);
  CHECK(oracle_attention(qkv, B, T, D, heads, 3, -1, ctx, NULL, vm) == 0);
  CHECK(oracle_attention(qkv, B, T, D, heads, T + 5, 2, ctx, sm, NULL) == 0);
  CHECK(oracle_attention(qkv, B, T, D, D + 1, -1, -1, ctx, NULL, NULL) == 2);
  for (size_t i = 0; i < n; ++i) CHECK(isfinite(ctx[i]));
  double *dq = need(3 * n * sizeof(double)), *mg = need(3 * n * sizeof(double));
  CHECK(oracle_attention_bwd(qkv, ctx, B, T, D, heads, -1, -1, dq, mg) == 0);
  CHECK(oracle_attention_bwd(qkv, ctx, B, T, D, heads, 2, 1, dq, NULL) == 0);
  CHECK(oracle_attention_bwd(qkv, ctx, B, T, D, D + 1, 2, 1, dq, NULL) == 2);
  for (size_t i = 0; i < 3 * n; ++i) CHECK(isfinite(dq[i]));
  /* the normalisation's backward on the same buffers: rows of D entries */
  oracle_layernorm_bwd(qkv, B * T, D, qkv, 1e-6, ctx, vm, dq, mg);
  oracle_layernorm_bwd(qkv, B * T, D, NULL, 1e-6, ctx, vm, NULL, NULL);
  free(qkv); free(ctx); free(vm); free(sm); free(dq); free(mg);
}

int main(void) {
  /* Fig. 2 rounds floor(t + 0.5): with 127 present the scale is exactly 1 */
  const float ties[8] = {127.0f, 0.5f, -0.5f, 1.5f, -1.5f, 2.5f, -2.5f, -127.0f};
  const int8_t want[8] = {127, 1, 0, 2, -1, 3, -2, -127};
  int8_t q[8];
  float s;
  CHECK(oracle_quantize(ties, 1, 8, 8, -1, q, &s, NULL) == 0);
  CHECK(s == 1.0f);
  for (int i = 0; i < 8; ++i) CHECK(q[i] == want[i]);
  const float seven[3] = {7.0f, -3.5f, 0.49f};
  CHECK(oracle_quantize(seven, 3, 1, 4, 0, q, &s, NULL) == 0);
  CHECK(s == 1.0f && q[0] == 7 && q[1] == -3 && q[2] == 0);
  const float bad[2] = {1.0f, INFINITY};
  CHECK(oracle_quantize(bad, 1, 2, 8, -1, q, &s, NULL) == 1);

  one_shape(1, 1, 1, 8, 8);
  one_shape(3, 5, 4, 8, 4);
  one_shape(7, 9, 5, 4, 4);
  one_shape(33, 17, 6, 8, 2);
  one_shape(2, 64, 3, 5, 8);
  one_conv(1, 1, 1, 1, 0);
  one_conv(2, 5, 3, 32, 15);
  one_conv(3, 40, 2, 15, 14);
  one_conv(1, 9, 4, 4, 0);
  one_attention(1, 1, 1, 1);
  one_attention(2, 7, 6, 3);
  one_attention(1, 33, 8, 2);
  printf("oracle sanitizer run ok\n");
  return 0;
}
