// Driver of the host emulation of the depthwise-convolution kernels: the test splices the kernels of
// paper_2203_15952_amd/csrc/conv.hip in front of this file (with hip_on_host.h in place of the HIP
// headers), every GPU thread of a block runs as an OS thread with real barriers, LDS is a heap block
// of exactly the launched size, and the build carries the address and undefined-behaviour sanitizers.
// Results are compared with plain float64 loops written here.
static float *mk(size_t n, float v, unsigned seed) { float *p = (float *)malloc(n * 4 + 4); uint32_t s = seed; for (size_t i = 0; i < n; ++i) { s = s * 1664525u + 1013904223u; p[i] = v * ((float)(s >> 8) / 8388608.0f - 1.0f); } return p; }
static int bad = 0;
static void cmp(const char *what, const float *got, const double *ref, const double *mag, size_t n) {
  double worst = 0;
  for (size_t i = 0; i < n; ++i) { double e = fabs((double)got[i] - ref[i]) / (mag[i] + 1e-30); if (e > worst) worst = e; }
  printf("  %-6s worst err / sum|terms| = %.3g\n", what, worst);
  if (!(worst < 1e-4)) bad = 1;
}
static void one(int64_t B, int64_t T, int64_t C, int kw, int pad) {
  printf("case %ld %ld %ld %d %d\n", (long)B, (long)T, (long)C, kw, pad); fflush(stdout);
  size_t n = B * T * C;
  float *x = mk(n, 1.0f, 1), *dout = mk(n, 0.1f, 2), *dfac = mk(n, 1.0f, 3), *w = mk((size_t)kw * C, 0.3f, 4), *bias = mk(C, 0.1f, 5);
  float *out = mk(n, 0, 0), *dx = mk(n, 0, 0), *dw = mk((size_t)kw * C, 0, 0), *db = mk(C, 0, 0);
  uint32_t am = 0;
  ConvGeom g = geom(B, T, C, kw, pad);
  unsigned blocks = g.cgroups * g.tgroups * B;
  std::vector<double> ref(n), mag(n);
  // forward, no activation
  if (kw <= kTapsMax) run(blocks, 256, (size_t)(kTile + 2 * kw - 1) * 256, [&] { dwconv_kernel(x, nullptr, w, bias, nullptr, nullptr, 0, 0, g, pad, out, nullptr, &am); });
  else run(8, 256, 0, [&] { dwconv_any_kernel(x, nullptr, w, bias, nullptr, nullptr, 0, 0, g, pad, out, nullptr, &am); });
  float mx = 0;
  for (int64_t b = 0; b < B; ++b) for (int64_t t = 0; t < T; ++t) for (int64_t c = 0; c < C; ++c) {
    double a = bias[c], m = fabs(a);
    for (int j = 0; j < kw; ++j) { int64_t u = t + j - pad; if (u < 0 || u >= T) continue; double pr = (double)w[j * C + c] * x[(b * T + u) * C + c]; a += pr; m += fabs(pr); }
    ref[(b * T + t) * C + c] = a; mag[(b * T + t) * C + c] = m;
  }
  cmp("fwd", out, ref.data(), mag.data(), n);
  for (size_t i = 0; i < n; ++i) mx = std::max(mx, fabsf(out[i]));
  if (__float_as_uint(mx) != am) { printf("  absmax mismatch\n"); bad = 1; }
  // dx
  if (kw <= kTapsMax) run(blocks, 256, (size_t)(kTile + 2 * kw - 1) * 256, [&] { dwconv_kernel(dout, dfac, w, nullptr, nullptr, nullptr, 0, 1, g, kw - 1 - pad, dx, nullptr, nullptr); });
  else run(8, 256, 0, [&] { dwconv_any_kernel(dout, dfac, w, nullptr, nullptr, nullptr, 0, 1, g, kw - 1 - pad, dx, nullptr, nullptr); });
  for (int64_t b = 0; b < B; ++b) for (int64_t u = 0; u < T; ++u) for (int64_t c = 0; c < C; ++c) {
    double a = 0, m = 0;
    for (int j = 0; j < kw; ++j) { int64_t t = u - j + pad; if (t < 0 || t >= T) continue; size_t at = (b * T + t) * C + c; double pr = (double)w[j * C + c] * ((double)dout[at] * dfac[at]); a += pr; m += fabs(pr); }
    ref[(b * T + u) * C + c] = a; mag[(b * T + u) * C + c] = m;
  }
  cmp("dx", dx, ref.data(), mag.data(), n);
  // dw, dbias
  int P = dw_partials(g);
  size_t pb = (size_t)P * (kw + 1) * C;
  float *part = mk(pb, 0, 0);
  int kwp = (kw + 3) & ~3;
  if (kw <= kTapsMax) run(g.cgroups * P, 256, (size_t)(2 * kTile + 2 * kwp + 6) * 256, [&] { dwconv_dw_kernel(dout, dfac, x, g, P, part); });
  else run(cdiv((int64_t)(kw + 1) * C, 256), 256, 0, [&] { dwconv_dw_any_kernel(dout, dfac, x, g, part); });
  run(cdiv((int64_t)(kw + 1) * C, 256), 256, 0, [&] { dwconv_dw_fold_kernel(part, P, kw, C, dw, db); });
  std::vector<double> rw((kw + 1) * C), mw((kw + 1) * C);
  for (int j = 0; j <= kw; ++j) for (int64_t c = 0; c < C; ++c) {
    double a = 0, m = 0;
    for (int64_t b = 0; b < B; ++b) for (int64_t t = 0; t < T; ++t) {
      size_t at = (b * T + t) * C + c; double dv = (double)dout[at] * dfac[at];
      if (j == kw) { a += dv; m += fabs(dv); continue; }
      int64_t u = t + j - pad; if (u < 0 || u >= T) continue;
      double pr = dv * x[(b * T + u) * C + c]; a += pr; m += fabs(pr);
    }
    rw[j * C + c] = a; mw[j * C + c] = m;
  }
  cmp("dw", dw, rw.data(), mw.data(), (size_t)kw * C);
  cmp("dbias", db, rw.data() + (size_t)kw * C, mw.data() + (size_t)kw * C, C);
  free(x); free(dout); free(dfac); free(w); free(bias); free(out); free(dx); free(dw); free(db); free(part);
}
}  // namespace
}  // namespace aqt
int main() {
  using namespace aqt;
  one(2, 37, 70, 15, 14); one(1, 5, 3, 32, 15); one(2, 50, 64, 40, 20); one(1, 100, 130, 1, 0); one(1, 1, 1, 1, 0);
  one(2, 129, 96, 16, 8); one(2, 128, 64, 17, 0); one(2, 19, 24, 32, 15); one(1, 200, 64, 32, 15); one(2, 65, 5, 31, 30);
  one(1, 64, 64, 3, 2);
  printf(bad ? "MISMATCH\n" : "ok\n"); return bad;
}
