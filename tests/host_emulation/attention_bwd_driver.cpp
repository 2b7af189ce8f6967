// Driver of the host emulation of the attention backward kernels (row-dot, dq, dk/dv) after the forward
// kernel has produced ctx and lse; spliced behind the kernels of attention.hip like attention_driver.cpp.
// Results are compared with plain float64 loops written here.
static int bad = 0;
static void one(int64_t B, int64_t T, int64_t D, int heads, int left, int right) {
  printf("case %ld %ld %ld %d %d %d\n", (long)B, (long)T, (long)D, heads, left, right); fflush(stdout);
  const size_t n = (size_t)(B * T * D);
  float *qkv = (float *)malloc(3 * n * 4), *ctx = (float *)malloc(n * 4), *dctx = (float *)malloc(n * 4);
  float *lse = (float *)malloc((size_t)(B * T * heads) * 4), *dsum = (float *)malloc((size_t)(B * T * heads) * 4);
  float *dqkv = (float *)malloc(3 * n * 4);
  uint32_t s = 11u;
  for (size_t i = 0; i < 3 * n; ++i) { s = s * 1664525u + 1013904223u; qkv[i] = 2.0f * ((float)(s >> 8) / 8388608.0f - 1.0f); dqkv[i] = NAN; }
  for (size_t i = 0; i < n; ++i) { s = s * 1664525u + 1013904223u; dctx[i] = (float)(s >> 8) / 8388608.0f - 1.0f; }
  AttnGeom g = attn_geom(B, T, D, heads, left, right);
  const unsigned blocks = (unsigned)(g.qtiles * heads * B);
  run(blocks, 256, 0, [&] { attention_fwd_kernel(qkv, g, ctx, nullptr, lse); });
  run((unsigned)cdiv(B * T, 4), 256, 0, [&] { attention_rowdot_kernel(dctx, ctx, g, dsum); });
  run(blocks, 256, 0, [&] { attention_bwd_dq_kernel(qkv, dctx, lse, dsum, g, dqkv); });
  run(blocks, 256, 0, [&] { attention_bwd_dkv_kernel(qkv, dctx, lse, dsum, g, dqkv); });
  const int dh = (int)(D / heads);
  const double scale = 1.0 / sqrt((double)dh);
  std::vector<double> ref(3 * n, 0.0), mag(3 * n, 0.0), p(T), dp(T);
  for (int64_t b = 0; b < B; ++b) for (int h = 0; h < heads; ++h) for (int64_t t = 0; t < T; ++t) {
    int64_t j0 = (left < 0 || t - left < 0) ? 0 : t - left, j1 = (right < 0 || t + right > T - 1) ? T - 1 : t + right;
    const size_t qo = (b * T + t) * 3 * D + h * dh;
    double m = -1e300, sum = 0, dd = 0, dda = 0;
    for (int64_t j = j0; j <= j1; ++j) { double a = 0; for (int d = 0; d < dh; ++d) a += (double)qkv[qo + d] * qkv[(b * T + j) * 3 * D + D + h * dh + d]; p[j] = a * scale; if (p[j] > m) m = p[j]; }
    for (int64_t j = j0; j <= j1; ++j) { p[j] = exp(p[j] - m); sum += p[j]; }
    for (int64_t j = j0; j <= j1; ++j) { double a = 0; for (int d = 0; d < dh; ++d) a += (double)dctx[(b * T + t) * D + h * dh + d] * qkv[(b * T + j) * 3 * D + 2 * D + h * dh + d]; p[j] /= sum; dp[j] = a; dd += p[j] * a; dda += p[j] * fabs(a); }
    for (int64_t j = j0; j <= j1; ++j) {
      const double ds = p[j] * (dp[j] - dd) * scale, dsa = p[j] * (fabs(dp[j]) + dda) * scale;
      const size_t ko = (b * T + j) * 3 * D + D + h * dh, vo = ko + D;
      for (int d = 0; d < dh; ++d) {
        ref[qo + d] += ds * qkv[ko + d]; mag[qo + d] += dsa * fabs(qkv[ko + d]);
        ref[ko + d] += ds * qkv[qo + d]; mag[ko + d] += dsa * fabs(qkv[qo + d]);
        const double gd = dctx[(b * T + t) * D + h * dh + d];
        ref[vo + d] += p[j] * gd; mag[vo + d] += p[j] * fabs(gd);
      }
    }
  }
  double worst = 0;
  for (size_t i = 0; i < 3 * n; ++i) { double e = fabs((double)dqkv[i] - ref[i]) / (mag[i] + 1e-30); if (!(e <= worst)) worst = e; }
  printf("  worst err / sum|terms| = %.3g\n", worst);
  if (!(worst < 1e-4)) { printf("  MISMATCH\n"); bad = 1; }
  free(qkv); free(ctx); free(dctx); free(lse); free(dsum); free(dqkv);
}
}  // namespace
}  // namespace aqt
int main() {
  using namespace aqt;
  one(1, 1, 1, 1, -1, -1); one(1, 70, 64, 1, -1, -1); one(1, 130, 36, 1, 23, 0); one(2, 65, 12, 3, 5, 7);
  one(1, 64, 8, 1, 0, 0);
  printf(bad ? "MISMATCH\n" : "ok\n"); return bad;
}
