// Driver of the host emulation of the attention kernel: the test splices the kernel of
// paper_2203_15952_amd/csrc/attention.hip in front of this file (hip_on_host.h in place of the HIP
// headers); every GPU thread of a block runs as an OS thread with real barriers under the address and
// undefined-behaviour sanitizers.  Results are compared with plain float64 loops written here.
static int bad = 0;
static void one(int64_t B, int64_t T, int64_t D, int heads, int left, int right) {
  printf("case %ld %ld %ld %d %d %d\n", (long)B, (long)T, (long)D, heads, left, right); fflush(stdout);
  const size_t n = (size_t)(B * T * D);
  float *qkv = (float *)malloc(3 * n * 4), *ctx = (float *)malloc(n * 4);
  uint32_t s = 7u, am = 0;
  for (size_t i = 0; i < 3 * n; ++i) { s = s * 1664525u + 1013904223u; qkv[i] = 2.0f * ((float)(s >> 8) / 8388608.0f - 1.0f); }
  AttnGeom g = attn_geom(B, T, D, heads, left, right);
  run((unsigned)(g.qtiles * heads * B), 256, 0, [&] { attention_fwd_kernel(qkv, g, ctx, &am, nullptr); });
  const int dh = (int)(D / heads);
  double worst = 0; float mx = 0;
  std::vector<double> p(T);
  for (int64_t b = 0; b < B; ++b) for (int64_t t = 0; t < T; ++t) for (int h = 0; h < heads; ++h) {
    int64_t j0 = (left < 0 || t - left < 0) ? 0 : t - left, j1 = (right < 0 || t + right > T - 1) ? T - 1 : t + right;
    double m = -1e300, sum = 0;
    for (int64_t j = j0; j <= j1; ++j) { double a = 0; for (int d = 0; d < dh; ++d) a += (double)qkv[(b * T + t) * 3 * D + h * dh + d] * qkv[(b * T + j) * 3 * D + D + h * dh + d]; p[j] = a / sqrt((double)dh); if (p[j] > m) m = p[j]; }
    for (int64_t j = j0; j <= j1; ++j) { p[j] = exp(p[j] - m); sum += p[j]; }
    for (int d = 0; d < dh; ++d) {
      double a = 0, ab = 0;
      for (int64_t j = j0; j <= j1; ++j) { double v = qkv[(b * T + j) * 3 * D + 2 * D + h * dh + d]; a += p[j] * v; ab += p[j] * fabs(v); }
      double e = fabs((double)ctx[(b * T + t) * D + h * dh + d] - a / sum) / (ab / sum + 1e-30);
      if (e > worst) worst = e;
    }
  }
  for (size_t i = 0; i < n; ++i) mx = std::max(mx, fabsf(ctx[i]));
  printf("  worst err / sum p|v| = %.3g\n", worst);
  if (!(worst < 1e-4) || __float_as_uint(mx) != am) { printf("  MISMATCH\n"); bad = 1; }
  free(qkv); free(ctx);
}
}  // namespace
}  // namespace aqt
int main() {
  using namespace aqt;
  one(1, 1, 1, 1, -1, -1); one(1, 70, 128, 2, -1, -1); one(1, 130, 72, 2, 23, 0); one(2, 65, 12, 3, 5, 7);
  one(1, 140, 64, 1, -1, 3); one(1, 64, 36, 1, 0, 0); one(1, 150, 8, 2, 70, 70);
  printf(bad ? "MISMATCH\n" : "ok\n"); return bad;
}
