// C ABI of libaqt: argument checks, workspace carving and dispatch.  Every entry
// point is declared and documented in include/aqt.h.
#include "aqt_internal.h"

namespace aqt {
thread_local int g_last_hip_error = 0;

namespace {

struct FwdWorkspace {
  float *partials;   // kMaxPartials abs-max slots
  uint32_t *wpart;   // kWeightSlabs x N per-channel slab maxima
  float *s_x;        // 1
  float *s_w;        // N
  int8_t *xq;        // M*K
  uint8_t *wq;       // packed weight operand
  uint8_t *wfrag;    // weights in MFMA-fragment order (scratch of the contraction)
  size_t total;
};

// Carve the training-forward workspace.  Buffers the caller keeps through
// `saved` are still laid out (simple, and the sizes stay shape-only).
FwdWorkspace carve_fwd(void *ws, int64_t M, int64_t K, int64_t N, int bits_w) {
  FwdWorkspace f;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  f.partials = reinterpret_cast<float *>(take(kMaxPartials * sizeof(float)));
  f.wpart = reinterpret_cast<uint32_t *>(take(weight_ws_bytes(N)));
  f.s_x = reinterpret_cast<float *>(take(sizeof(float)));
  f.s_w = reinterpret_cast<float *>(take(static_cast<size_t>(N) * sizeof(float)));
  f.xq = reinterpret_cast<int8_t *>(take(static_cast<size_t>(M) * K));
  f.wq = take(aqt_packed_weight_bytes(K, N, bits_w));
  f.wfrag = take(fwd_q_workspace_bytes(K, N));
  f.total = off;
  return f;
}

bool shape_ok(int64_t a, int64_t b) { return a >= 1 && b >= 1; }

struct FfnWorkspace {
  void *ln;          // layer-normalisation scratch
  uint32_t *wpart1;  // per-channel slab maxima, first / second weight matrix
  uint32_t *wpart2;
  void *wfrag1;      // weights in MFMA-fragment order (also large enough for the weight-only forward)
  void *wfrag2;
  float *h_absmax;   // max|h| emitted by the first contraction
  size_t total;
};

FfnWorkspace carve_ffn_fwd(void *ws, int64_t M, int64_t D, int64_t H) {
  FfnWorkspace f;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  f.ln = take(layernorm_ws_bytes(M));
  f.wpart1 = reinterpret_cast<uint32_t *>(take(weight_ws_bytes(H)));
  f.wpart2 = reinterpret_cast<uint32_t *>(take(weight_ws_bytes(D)));
  const size_t frag = fwd_wonly_workspace_bytes(D, H);   // 2 bytes per weight covers both forward kinds
  f.wfrag1 = take(frag);
  f.wfrag2 = take(frag);
  f.h_absmax = reinterpret_cast<float *>(take(sizeof(float)));
  f.total = off;
  return f;
}

// Backward of the feed-forward module: one dense-backward workspace large enough for either
// layer, reused, plus the gradient with respect to h, [M,H].
size_t ffn_bwd_ws(int64_t M, int64_t D, int64_t H) {
  const size_t a = bwd_workspace_bytes(M, D, H), b = bwd_workspace_bytes(M, H, D);
  return (a > b ? a : b) + align_up(static_cast<size_t>(M) * H * sizeof(float), 256);
}

// Backward of the convolution module: one dense-backward workspace large enough for either
// pointwise layer, then the gradients with respect to s and g [M,D] each, the gradient in front
// of the GLU [M,2D], and the partial sums of the depthwise taps.
struct ConvBwdWorkspace {
  size_t core;
  float *ds, *dg, *dv;
  void *taps;
  size_t total;
};

ConvBwdWorkspace carve_conv_bwd(void *ws, int64_t B, int64_t T, int64_t D, int kw) {
  ConvBwdWorkspace f;
  const int64_t M = B * T;
  const size_t a = bwd_workspace_bytes(M, D, 2 * D), b = bwd_workspace_bytes(M, D, D);
  f.core = a > b ? a : b;
  size_t off = f.core;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  const size_t md = static_cast<size_t>(M) * D * sizeof(float);
  f.ds = reinterpret_cast<float *>(take(md));
  f.dg = reinterpret_cast<float *>(take(md));
  f.dv = reinterpret_cast<float *>(take(2 * md));
  f.taps = take(dwconv_bwd_ws_bytes(D, kw));
  f.total = off;
  return f;
}

// Backward of the self-attention module: one dense-backward workspace for either projection, the
// gradients with respect to ctx [M,D] and qkv [M,3D], the attention backward's row sums.
struct MhsaBwdWorkspace {
  size_t core;
  float *dctx, *dqkv;
  void *att;
  size_t total;
};

MhsaBwdWorkspace carve_mhsa_bwd(void *ws, int64_t M, int64_t D, int heads) {
  MhsaBwdWorkspace f;
  const size_t a = bwd_workspace_bytes(M, D, 3 * D), b = bwd_workspace_bytes(M, D, D);
  f.core = a > b ? a : b;
  size_t off = f.core;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  const size_t md = static_cast<size_t>(M) * D * sizeof(float);
  f.dctx = reinterpret_cast<float *>(take(md));
  f.dqkv = reinterpret_cast<float *>(take(3 * md));
  f.att = take(attention_bwd_ws_bytes(1, M, heads));
  f.total = off;
  return f;
}

// Backward of the encoder layer: the largest module-backward workspace, then the gradient of the residual
// stream (two buffers, alternating), a module-input gradient, and the normalisation backward's partials.
struct LayerBwdWorkspace {
  size_t module;
  float *da, *db, *dm;
  void *ln;
  size_t total;
};

size_t conv_bwd_total(int64_t M, int64_t D, int kw);

LayerBwdWorkspace carve_layer_bwd(void *ws, int64_t M, int64_t D, int64_t H, int heads, int kw) {
  LayerBwdWorkspace f;
  size_t m = ffn_bwd_ws(M, D, H);
  const size_t a = carve_mhsa_bwd(nullptr, M, D, heads).total, c = conv_bwd_total(M, D, kw);
  if (a > m) m = a;
  if (c > m) m = c;
  f.module = m;
  size_t off = m;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  const size_t md = static_cast<size_t>(M) * D * sizeof(float);
  f.da = reinterpret_cast<float *>(take(md));
  f.db = reinterpret_cast<float *>(take(md));
  f.dm = reinterpret_cast<float *>(take(md));
  f.ln = take(layernorm_bwd_ws_bytes(D));
  f.total = off;
  return f;
}

bool conv_shape_ok(int64_t B, int64_t T, int64_t C, int kw, int pad_left) {
  return B >= 1 && T >= 1 && C >= 1 && kw >= 1 && kw <= 4096 && pad_left >= 0 && pad_left < kw &&
         B <= (int64_t(1) << 40) / T;
}

size_t conv_bwd_total(int64_t M, int64_t D, int kw) { return carve_conv_bwd(nullptr, 1, M, D, kw).total; }

bool policy_ok(const aqt_dense_policy &p) {
  return bits_ok(p.bits_w) && (p.bits_x == 0 || bits_ok(p.bits_x)) && (p.weights_ready == 0 || p.weights_ready == 1);
}

// The weight side of one dense layer inside a module call.  Training: quantize w now (the quantizer
// also emits the matrix-core operand into `wfrag` when the contraction kernel takes one).  Serving
// (weights_ready): nothing to do; the prepared operand of the layer is used if there is one.
// A module called inside a layer: its input is x + alpha * m (the residual stream plus the previous module's
// output), formed by the module's normalisation pass and left in r_out.
struct ResidualIn {
  const float *m;
  float alpha;
  float *r_out;
};

struct WeightSide {
  void *operand;   // what launch_dense_fwd_q gets as its workspace
  bool prepared;   // whether it already holds the matrix-core operand
};
// With a job list the quantizer launch is left to the caller (launch_quantize_weights_group over the list).
struct WeightJobList {
  WeightJob job[kWeightJobsMax];
  int n = 0;
};
aqt_status weight_side(const aqt_dense_policy &p, const float *w, const aqt_saved &l, int64_t M, int64_t K, int64_t N,
                       int epilogue, uint32_t *wpart, void *wfrag, hipStream_t st, int32_t *dev_status,
                       WeightSide *out, WeightJobList *later = nullptr) {
  const bool takes = p.bits_x && fwd_q_takes_fragments(M, K, N, epilogue) && reinterpret_cast<uintptr_t>(l.xq) % 16 == 0;
  if (p.weights_ready) {
    const bool have = takes && l.wprep && reinterpret_cast<uintptr_t>(l.wprep) % 16 == 0;
    out->operand = have ? l.wprep : wfrag;
    out->prepared = have;
    return AQT_OK;
  }
  if (!w) return AQT_ERR_INVALID_ARG;
  out->operand = wfrag;
  out->prepared = takes;
  if (later) {
    if (later->n >= kWeightJobsMax) return AQT_ERR_INVALID_ARG;
    later->job[later->n++] = WeightJob{w, K, N, p.bits_w, l.wq_packed, l.s_w, l.wq_kn, l.mask_w, wpart,
                                       takes ? wfrag : nullptr};
    return AQT_OK;
  }
  return launch_quantize_weights(w, K, N, p.bits_w, l.wq_packed, l.s_w, l.wq_kn, l.mask_w, wpart, st, dev_status,
                                 takes ? wfrag : nullptr);
}

// The weight-side buffers of an encoder layer's eight dense layers, behind the modules' shared workspace: the layer
// call quantizes all of its matrices in one launch pair before the first module runs.
struct LayerFwdWorkspace {
  size_t module;           // bytes the modules share, at the front
  uint32_t *wpart[8];
  void *wfrag[8];
  size_t total;
};
LayerFwdWorkspace carve_layer_fwd(void *ws, int64_t M, int64_t D, int64_t H) {
  LayerFwdWorkspace f;
  const size_t a = carve_ffn_fwd(nullptr, M, D, H).total, b = carve_ffn_fwd(nullptr, M, D, 3 * D).total;
  f.module = a > b ? a : b;          // 3 D covers the convolution module's 2 D as well
  size_t off = f.module;
  auto take = [&](size_t bytes) {
    uint8_t *p = ws ? static_cast<uint8_t *>(ws) + off : nullptr;
    off += align_up(bytes, 256);
    return p;
  };
  // fan-in, fan-out in aqt_layer_policy order
  const int64_t kn[8][2] = {{D, H}, {H, D}, {D, 3 * D}, {D, D}, {D, 2 * D}, {D, D}, {D, H}, {H, D}};
  for (int i = 0; i < 8; ++i) {
    f.wpart[i] = reinterpret_cast<uint32_t *>(take(weight_ws_bytes(kn[i][1])));
    f.wfrag[i] = take(fwd_wonly_workspace_bytes(kn[i][0], kn[i][1]));
  }
  f.total = off;
  return f;
}

// The int32 accumulator must hold K * qmax_x * qmax_w; packed (<= 4 bit) weights enter the
// matrix cores as 16 * code, so their sums carry a factor 16 until the final shift.
bool acc_fits(int64_t K, int bits_x, int bits_w) {
  const int64_t lim = (int64_t(1) << 31) / (packed4(bits_w) ? 16 : 1);
  return K * qmax_of(bits_x) * qmax_of(bits_w) < lim;
}

}  // namespace
}  // namespace aqt

using namespace aqt;

// Every argument check of the feed-forward module's forward, so that a caller of several modules can run all of
// them before the first launch.
static aqt_status ffn_fwd_check(const float *x, float ln_eps, const float *w1, const float *w2, int64_t M, int64_t D,
                                int64_t H, const aqt_dense_policy *policy, const float *y, const aqt_ffn_saved *saved,
                                const void *ws, size_t ws_bytes) {
  if (!x || !y || !policy || !saved || !shape_ok(M, D) || H < 1 || !(ln_eps >= 0.0f)) return AQT_ERR_INVALID_ARG;
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  if (!policy_ok(p1) || !policy_ok(p2)) return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->l1, &l2 = saved->l2;
  if (!saved->h || !l1.wq_packed || !l1.s_w || !l2.wq_packed || !l2.s_w) return AQT_ERR_INVALID_ARG;
  if ((!p1.weights_ready && !w1) || (!p2.weights_ready && !w2)) return AQT_ERR_INVALID_ARG;
  if (p1.bits_x ? (!l1.xq || !l1.s_x) : !saved->xn) return AQT_ERR_INVALID_ARG;
  if (p2.bits_x && (!l2.xq || !l2.s_x)) return AQT_ERR_INVALID_ARG;
  if (p1.bits_x && !acc_fits(D, p1.bits_x, p1.bits_w)) return AQT_ERR_UNSUPPORTED;
  if (p2.bits_x && !acc_fits(H, p2.bits_x, p2.bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < carve_ffn_fwd(nullptr, M, D, H).total) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

static aqt_status ffn_fwd_impl(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps, const float *w1,
                       const float *b1, const float *w2, const float *b2, int64_t M, int64_t D, int64_t H,
                       const aqt_dense_policy *policy, float *y, const aqt_ffn_saved *saved, void *ws,
                       size_t ws_bytes, void *stream, int32_t *dev_status, const ResidualIn *res,
    const WeightSide *sides = nullptr) {
  AQT_TRY(ffn_fwd_check(x, ln_eps, w1, w2, M, D, H, policy, y, saved, ws, ws_bytes));
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  const aqt_saved &l1 = saved->l1, &l2 = saved->l2;
  FfnWorkspace f = carve_ffn_fwd(ws, M, D, H);
  hipStream_t st = static_cast<hipStream_t>(stream);

  // normalisation (+ first quantizer), first weights, first contraction with Swish
  WeightSide s1, s2;
  if (sides) {
    s1 = sides[0];
    s2 = sides[1];
  } else {   // both matrices through the weight quantizer in one launch pair
    WeightJobList jobs;
    AQT_TRY(weight_side(p1, w1, l1, M, D, H, AQT_EPI_SWISH, f.wpart1, f.wfrag1, st, dev_status, &s1, &jobs));
    AQT_TRY(weight_side(p2, w2, l2, M, H, D, AQT_EPI_NONE, f.wpart2, f.wfrag2, st, dev_status, &s2, &jobs));
    AQT_TRY(launch_quantize_weights_group(jobs.job, jobs.n, st, dev_status));
  }
  const bool want_absmax = p2.bits_x != 0;
  if (p1.bits_x) {
    // the normalisation's first pass also clears the word the contraction's epilogue collects max|h| in
    uint32_t *hmax = want_absmax ? reinterpret_cast<uint32_t *>(f.h_absmax) : nullptr;
    AQT_TRY(launch_layernorm_quantize(x, M, D, ln_gamma, ln_beta, ln_eps, p1.bits_x, l1.xq, l1.s_x, saved->xn,
                                      saved->row_stats, f.ln, st, dev_status, res ? res->m : nullptr,
                                      res ? res->alpha : 0.0f, res ? res->r_out : nullptr, hmax));
    AQT_TRY(launch_dense_fwd_q(l1.xq, l1.s_x, l1.wq_packed, l1.s_w, M, D, H, p1.bits_w, b1, AQT_EPI_SWISH, saved->h,
                               nullptr, hmax, s1.operand, st, l1.dact, s1.prepared, true));
  } else {
    AQT_TRY(launch_layernorm_quantize(x, M, D, ln_gamma, ln_beta, ln_eps, 8, nullptr, nullptr, saved->xn,
                                      saved->row_stats, f.ln, st, dev_status, res ? res->m : nullptr,
                                      res ? res->alpha : 0.0f, res ? res->r_out : nullptr));
    AQT_TRY(launch_dense_fwd_wonly(saved->xn, l1.wq_packed, l1.s_w, M, D, H, p1.bits_w, b1, AQT_EPI_SWISH, saved->h,
                                   f.wfrag1, st));
  }
  // second quantizer (one pass when the producer emitted max|h|), second contraction
  if (p2.bits_x) {
    if (p1.bits_x) {
      AQT_TRY(launch_quantize_with_absmax(saved->h, M, H, H, p2.bits_x, reinterpret_cast<const uint32_t *>(f.h_absmax),
                                          l2.xq, l2.s_x, l2.mask_x, st, dev_status));
    } else {
      AQT_TRY(launch_quantize(saved->h, M, H, H, p2.bits_x, AQT_AXIS_ALL, l2.xq, l2.s_x, l2.mask_x,
                              static_cast<float *>(f.ln), st, dev_status));
    }
    return launch_dense_fwd_q(l2.xq, l2.s_x, l2.wq_packed, l2.s_w, M, H, D, p2.bits_w, b2, AQT_EPI_NONE, y, nullptr,
                              nullptr, s2.operand, st, nullptr, s2.prepared);
  }
  return launch_dense_fwd_wonly(saved->h, l2.wq_packed, l2.s_w, M, H, D, p2.bits_w, b2, AQT_EPI_NONE, y, f.wfrag2, st);
}

static aqt_status conv_module_fwd_check(const float *x, float ln_eps, const float *w1, const float *w_dw,
                                        const float *w2, int64_t B, int64_t T, int64_t D, int kw, int pad_left,
                                        const aqt_dense_policy *policy, const float *y, const aqt_conv_saved *saved,
                                        const void *ws, size_t ws_bytes) {
  if (!x || !w_dw || !y || !policy || !saved || !conv_shape_ok(B, T, D, kw, pad_left) || !(ln_eps >= 0.0f))
    return AQT_ERR_INVALID_ARG;
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  if (!policy_ok(p1) || !policy_ok(p2) || p1.bits_x == 0 || p2.bits_x == 0) return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->pw1, &l2 = saved->pw2;
  if (!saved->g || !saved->s || !l1.xq || !l1.s_x || !l1.wq_packed || !l1.s_w || !l2.xq || !l2.s_x ||
      !l2.wq_packed || !l2.s_w)
    return AQT_ERR_INVALID_ARG;
  if ((!p1.weights_ready && !w1) || (!p2.weights_ready && !w2)) return AQT_ERR_INVALID_ARG;
  if (!acc_fits(D, p1.bits_x, p1.bits_w) || !acc_fits(D, p2.bits_x, p2.bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < carve_ffn_fwd(nullptr, B * T, D, 2 * D).total) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

static aqt_status conv_module_fwd_impl(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps,
                               const float *w1, const float *b1, const float *w_dw, const float *b_dw,
                               const float *norm_scale, const float *norm_shift, const float *w2, const float *b2,
                               int64_t B, int64_t T, int64_t D, int kw, int pad_left, const aqt_dense_policy *policy,
                               float *y, const aqt_conv_saved *saved, void *ws, size_t ws_bytes, void *stream,
                               int32_t *dev_status, const ResidualIn *res,
    const WeightSide *sides = nullptr) {
  AQT_TRY(conv_module_fwd_check(x, ln_eps, w1, w_dw, w2, B, T, D, kw, pad_left, policy, y, saved, ws, ws_bytes));
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  const aqt_saved &l1 = saved->pw1, &l2 = saved->pw2;
  const int64_t M = B * T;
  FfnWorkspace f = carve_ffn_fwd(ws, M, D, 2 * D);
  hipStream_t st = static_cast<hipStream_t>(stream);

  // normalisation + first quantizer, first pointwise convolution with the GLU
  WeightSide s1, s2;
  if (sides) {
    s1 = sides[0];
    s2 = sides[1];
  } else {
    WeightJobList jobs;
    AQT_TRY(weight_side(p1, w1, l1, M, D, 2 * D, AQT_EPI_GLU, f.wpart1, f.wfrag1, st, dev_status, &s1, &jobs));
    AQT_TRY(weight_side(p2, w2, l2, M, D, D, AQT_EPI_NONE, f.wpart2, f.wfrag2, st, dev_status, &s2, &jobs));
    AQT_TRY(launch_quantize_weights_group(jobs.job, jobs.n, st, dev_status));
  }
  uint32_t *smax = reinterpret_cast<uint32_t *>(f.h_absmax);   // cleared by the normalisation's first pass
  AQT_TRY(launch_layernorm_quantize(x, M, D, ln_gamma, ln_beta, ln_eps, p1.bits_x, l1.xq, l1.s_x, nullptr,
                                    saved->row_stats, f.ln, st, dev_status, res ? res->m : nullptr,
                                    res ? res->alpha : 0.0f, res ? res->r_out : nullptr, smax));
  AQT_TRY(launch_dense_fwd_q(l1.xq, l1.s_x, l1.wq_packed, l1.s_w, M, D, 2 * D, p1.bits_w, b1, AQT_EPI_GLU, saved->g,
                             nullptr, nullptr, s1.operand, st, l1.dact, s1.prepared));
  // depthwise convolution, normalisation, Swish; max|s| for the one-pass quantizer
  AQT_TRY(launch_dwconv_fwd(saved->g, w_dw, b_dw, norm_scale, norm_shift, 1, B, T, D, kw, pad_left, saved->s,
                            saved->dfac, smax, st, true));
  // second pointwise convolution
  AQT_TRY(launch_quantize_with_absmax(saved->s, M, D, D, p2.bits_x, reinterpret_cast<const uint32_t *>(f.h_absmax),
                                      l2.xq, l2.s_x, l2.mask_x, st, dev_status));
  return launch_dense_fwd_q(l2.xq, l2.s_x, l2.wq_packed, l2.s_w, M, D, D, p2.bits_w, b2, AQT_EPI_NONE, y, nullptr,
                            nullptr, s2.operand, st, nullptr, s2.prepared);
}

static aqt_status mhsa_fwd_check(const float *x, float ln_eps, const float *wqkv, const float *wo, int64_t B,
                                 int64_t T, int64_t D, int heads, const aqt_dense_policy *policy, const float *y,
                                 const aqt_mhsa_saved *saved, const void *ws, size_t ws_bytes) {
  if (!x || !y || !policy || !saved || B < 1 || T < 1 || D < 1 || heads < 1 || D % heads || !(ln_eps >= 0.0f))
    return AQT_ERR_INVALID_ARG;
  if (!attention_shape_ok(B, T, D, heads)) return AQT_ERR_UNSUPPORTED;
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  if (!policy_ok(p1) || !policy_ok(p2) || p1.bits_x == 0 || p2.bits_x == 0) return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->qkv, &l2 = saved->out;
  if (!saved->qkv_f || !saved->ctx || !l1.xq || !l1.s_x || !l1.wq_packed || !l1.s_w || !l2.xq || !l2.s_x ||
      !l2.wq_packed || !l2.s_w)
    return AQT_ERR_INVALID_ARG;
  if ((!p1.weights_ready && !wqkv) || (!p2.weights_ready && !wo)) return AQT_ERR_INVALID_ARG;
  if (!acc_fits(D, p1.bits_x, p1.bits_w) || !acc_fits(D, p2.bits_x, p2.bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < carve_ffn_fwd(nullptr, B * T, D, 3 * D).total) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

static aqt_status mhsa_fwd_impl(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps, const float *wqkv,
                        const float *bqkv, const float *wo, const float *bo, int64_t B, int64_t T, int64_t D,
                        int heads, int left_context, int right_context, const aqt_dense_policy *policy, float *y,
                        const aqt_mhsa_saved *saved, void *ws, size_t ws_bytes, void *stream, int32_t *dev_status, const ResidualIn *res,
    const WeightSide *sides = nullptr) {
  AQT_TRY(mhsa_fwd_check(x, ln_eps, wqkv, wo, B, T, D, heads, policy, y, saved, ws, ws_bytes));
  const aqt_dense_policy p1 = policy[0], p2 = policy[1];
  const aqt_saved &l1 = saved->qkv, &l2 = saved->out;
  const int64_t M = B * T;
  FfnWorkspace f = carve_ffn_fwd(ws, M, D, 3 * D);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // normalisation + first quantizer, fused projection of queries, keys and values
  WeightSide s1, s2;
  if (sides) {
    s1 = sides[0];
    s2 = sides[1];
  } else {
    WeightJobList jobs;
    AQT_TRY(weight_side(p1, wqkv, l1, M, D, 3 * D, AQT_EPI_NONE, f.wpart1, f.wfrag1, st, dev_status, &s1, &jobs));
    AQT_TRY(weight_side(p2, wo, l2, M, D, D, AQT_EPI_NONE, f.wpart2, f.wfrag2, st, dev_status, &s2, &jobs));
    AQT_TRY(launch_quantize_weights_group(jobs.job, jobs.n, st, dev_status));
  }
  uint32_t *cmax = reinterpret_cast<uint32_t *>(f.h_absmax);   // cleared by the normalisation's first pass
  AQT_TRY(launch_layernorm_quantize(x, M, D, ln_gamma, ln_beta, ln_eps, p1.bits_x, l1.xq, l1.s_x, nullptr,
                                    saved->row_stats, f.ln, st, dev_status, res ? res->m : nullptr,
                                    res ? res->alpha : 0.0f, res ? res->r_out : nullptr, cmax));
  AQT_TRY(launch_dense_fwd_q(l1.xq, l1.s_x, l1.wq_packed, l1.s_w, M, D, 3 * D, p1.bits_w, bqkv, AQT_EPI_NONE,
                             saved->qkv_f, nullptr, nullptr, s1.operand, st, nullptr, s1.prepared));
  // attention in float32; max|ctx| for the one-pass quantizer
  AQT_TRY(launch_attention(saved->qkv_f, B, T, D, heads, left_context, right_context, saved->ctx, cmax, saved->lse,
                           st, true));
  // output projection
  AQT_TRY(launch_quantize_with_absmax(saved->ctx, M, D, D, p2.bits_x, reinterpret_cast<const uint32_t *>(f.h_absmax),
                                      l2.xq, l2.s_x, l2.mask_x, st, dev_status));
  return launch_dense_fwd_q(l2.xq, l2.s_x, l2.wq_packed, l2.s_w, M, D, D, p2.bits_w, bo, AQT_EPI_NONE, y, nullptr,
                            nullptr, s2.operand, st, nullptr, s2.prepared);
}

// Argument checks of the three module backward calls, each in one function so that the layer backward can run all
// of them before its first launch.
static aqt_status ffn_bwd_check(const float *dy, const aqt_ffn_saved *saved, int64_t M, int64_t D, int64_t H,
                                const aqt_dense_policy *policy, const float *dxn, const float *dw1, const float *dw2,
                                const void *ws, size_t ws_bytes) {
  if (!dy || !saved || !policy || !shape_ok(M, D) || H < 1) return AQT_ERR_INVALID_ARG;
  if (!policy_ok(policy[0]) || !policy_ok(policy[1])) return AQT_ERR_UNSUPPORTED;
  if (policy[0].bits_x == 0 || policy[1].bits_x == 0) return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->l1, &l2 = saved->l2;
  if (!l1.s_x || !l1.s_w || !l2.s_x || !l2.s_w || !l2.wq_kn || !l1.dact) return AQT_ERR_INVALID_ARG;
  if ((dxn && !l1.wq_kn) || (dw1 && !l1.xq) || (dw2 && !l2.xq)) return AQT_ERR_INVALID_ARG;
  if (!ws || ws_bytes < ffn_bwd_ws(M, D, H)) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

static aqt_status conv_module_bwd_check(const float *dy, const aqt_conv_saved *saved, const float *w_dw, int64_t B,
                                        int64_t T, int64_t D, int kw, int pad_left, const aqt_dense_policy *policy,
                                        const float *dxn, const float *dw1, const float *dw2, const void *ws,
                                        size_t ws_bytes) {
  if (!dy || !saved || !w_dw || !policy || !conv_shape_ok(B, T, D, kw, pad_left)) return AQT_ERR_INVALID_ARG;
  if (!policy_ok(policy[0]) || !policy_ok(policy[1])) return AQT_ERR_UNSUPPORTED;
  if (policy[0].bits_x == 0 || policy[1].bits_x == 0) return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->pw1, &l2 = saved->pw2;
  if (!l1.s_x || !l1.s_w || !l2.s_x || !l2.s_w || !l2.wq_kn || !l1.dact || !saved->dfac || !saved->g)
    return AQT_ERR_INVALID_ARG;
  if ((dxn && !l1.wq_kn) || (dw1 && !l1.xq) || (dw2 && !l2.xq)) return AQT_ERR_INVALID_ARG;
  if (!ws || ws_bytes < carve_conv_bwd(nullptr, B, T, D, kw).total) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

static aqt_status mhsa_bwd_check(const float *dy, const aqt_mhsa_saved *saved, int64_t B, int64_t T, int64_t D,
                                 int heads, const aqt_dense_policy *policy, const float *dxn, const float *dwqkv,
                                 const float *dwo, const void *ws, size_t ws_bytes) {
  if (!dy || !saved || !policy || B < 1 || T < 1 || D < 1 || heads < 1 || D % heads) return AQT_ERR_INVALID_ARG;
  if (!attention_shape_ok(B, T, D, heads)) return AQT_ERR_UNSUPPORTED;
  if (!policy_ok(policy[0]) || !policy_ok(policy[1]) || policy[0].bits_x == 0 || policy[1].bits_x == 0)
    return AQT_ERR_UNSUPPORTED;
  const aqt_saved &l1 = saved->qkv, &l2 = saved->out;
  if (!saved->lse || !saved->qkv_f || !saved->ctx || !l1.s_x || !l1.s_w || !l2.s_x || !l2.s_w || !l2.wq_kn)
    return AQT_ERR_INVALID_ARG;
  if ((dxn && !l1.wq_kn) || (dwqkv && !l1.xq) || (dwo && !l2.xq)) return AQT_ERR_INVALID_ARG;
  if (!ws || ws_bytes < carve_mhsa_bwd(nullptr, B * T, D, heads).total) return AQT_ERR_WORKSPACE;
  return AQT_OK;
}

extern "C" {

const char *aqt_status_string(aqt_status s) {
  switch (s) {
    case AQT_OK: return "ok";
    case AQT_ERR_INVALID_ARG: return "invalid argument";
    case AQT_ERR_UNSUPPORTED: return "unsupported configuration";
    case AQT_ERR_WORKSPACE: return "workspace missing or too small";
    case AQT_ERR_HIP: return "HIP runtime error";
    case AQT_ERR_NONFINITE: return "non-finite input";
    case AQT_ERR_SCRATCH: return "shape needs more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

int aqt_last_hip_error(void) { return g_last_hip_error; }

int aqt_version(void) { return 201; }

size_t aqt_packed_weight_bytes(int64_t K, int64_t N, int bits_w) {
  if (!shape_ok(K, N) || !bits_ok(bits_w)) return 0;
  return static_cast<size_t>(N) * static_cast<size_t>(packed4(bits_w) ? (K + 1) / 2 : K);
}

size_t aqt_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w) {
  (void)bits_x;
  switch (op) {
    case AQT_OP_QUANTIZE: return kMaxPartials * sizeof(float);
    case AQT_OP_QUANTIZE_WEIGHTS: return N >= 1 ? weight_ws_bytes(N) : 0;
    case AQT_OP_DENSE_FWD_WONLY: return (K >= 1 && N >= 1) ? fwd_wonly_workspace_bytes(K, N) : 0;
    case AQT_OP_DENSE_FWD_Q: return (K >= 1 && N >= 1) ? fwd_q_workspace_bytes(K, N) : 0;
    case AQT_OP_DENSE_FWD:
      if (!shape_ok(M, K) || N < 1 || !bits_ok(bits_w)) return 0;
      return carve_fwd(nullptr, M, K, N, bits_w).total;
    case AQT_OP_DENSE_BWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return bwd_workspace_bytes(M, K, N);
    case AQT_OP_DENSE_BWD_EPI:
      if (!shape_ok(M, K) || N < 1) return 0;
      return bwd_workspace_bytes(M, K, N) + align_up(static_cast<size_t>(M) * N * sizeof(float), 256);
    case AQT_OP_LAYERNORM_QUANTIZE: return M >= 1 ? layernorm_ws_bytes(M) : 0;
    case AQT_OP_FFN_FWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return carve_ffn_fwd(nullptr, M, K, N).total;
    case AQT_OP_FFN_BWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return ffn_bwd_ws(M, K, N);
    case AQT_OP_DEPTHWISE_CONV_BWD:
      if (!shape_ok(M, K) || N < 1 || N > 4096) return 0;
      return dwconv_bwd_ws_bytes(K, static_cast<int>(N));
    case AQT_OP_CONV_MODULE_FWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return carve_ffn_fwd(nullptr, M, K, 2 * K).total;
    case AQT_OP_MHSA_FWD:
      if (!shape_ok(M, K)) return 0;
      return carve_ffn_fwd(nullptr, M, K, 3 * K).total;
    case AQT_OP_CONFORMER_LAYER_FWD: {
      if (!shape_ok(M, K) || N < 1) return 0;
      return carve_layer_fwd(nullptr, M, K, N).total;
    }
    case AQT_OP_ATTENTION_BWD:
      if (M < 1 || N < 1) return 0;
      return attention_bwd_ws_bytes(1, M, static_cast<int>(N));
    case AQT_OP_LAYERNORM_BWD: return (M >= 1 && K >= 1) ? layernorm_bwd_ws_bytes(K) : 0;
    case AQT_OP_MHSA_BWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return carve_mhsa_bwd(nullptr, M, K, static_cast<int>(N)).total;
    case AQT_OP_CONFORMER_LAYER_BWD:
      if (!shape_ok(M, K) || N < 1) return 0;
      return carve_layer_bwd(nullptr, M, K, N, 64, 32).total;
    case AQT_OP_CONV_MODULE_BWD:
      if (!shape_ok(M, K) || N < 1 || N > 4096) return 0;
      return carve_conv_bwd(nullptr, 1, M, K, static_cast<int>(N)).total;
    default: return 0;
  }
}

aqt_status aqt_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int axis, int8_t *q,
                        float *scale, uint32_t *clip_mask, void *ws, size_t ws_bytes, void *stream,
                        int32_t *dev_status) {
  if (!x || !q || !scale || !shape_ok(rows, cols) || ldx < cols) return AQT_ERR_INVALID_ARG;
  if (axis != AQT_AXIS_ALL && axis != AQT_AXIS_ROWS && axis != AQT_AXIS_COLS) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits)) return AQT_ERR_UNSUPPORTED;
  if (axis == AQT_AXIS_ALL && (!ws || ws_bytes < kMaxPartials * sizeof(float))) return AQT_ERR_WORKSPACE;
  return launch_quantize(x, rows, cols, ldx, bits, axis, q, scale, clip_mask, static_cast<float *>(ws),
                         static_cast<hipStream_t>(stream), dev_status);
}

aqt_status aqt_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int axis,
                                   const float *scale, int8_t *q, uint32_t *clip_mask, void *stream) {
  if (!x || !q || !scale || !shape_ok(rows, cols) || ldx < cols) return AQT_ERR_INVALID_ARG;
  if (axis != AQT_AXIS_ALL && axis != AQT_AXIS_ROWS && axis != AQT_AXIS_COLS) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits)) return AQT_ERR_UNSUPPORTED;
  return launch_quantize_with_scale(x, rows, cols, ldx, bits, axis, scale, q, clip_mask,
                                    static_cast<hipStream_t>(stream));
}

aqt_status aqt_quantize_weights(const float *w, int64_t K, int64_t N, int bits_w, void *wq_packed, float *s_w,
                                int8_t *wq_kn, uint32_t *clip_mask_w, void *ws, size_t ws_bytes, void *stream,
                                int32_t *dev_status) {
  if (!w || !wq_packed || !s_w || !shape_ok(K, N)) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < weight_ws_bytes(N)) return AQT_ERR_WORKSPACE;
  return launch_quantize_weights(w, K, N, bits_w, wq_packed, s_w, wq_kn, clip_mask_w,
                                 static_cast<uint32_t *>(ws), static_cast<hipStream_t>(stream), dev_status);
}

aqt_status aqt_unpack_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, int8_t *codes_kn,
                              void *stream) {
  if (!wq_packed || !codes_kn || !shape_ok(K, N)) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  return launch_unpack_weights(wq_packed, K, N, bits_w, codes_kn, static_cast<hipStream_t>(stream));
}

aqt_status aqt_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                           int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                           int epilogue, float *y, int32_t *acc_out, void *ws, size_t ws_bytes, void *stream) {
  if (!xq || !s_x || !wq_packed || !s_w || !y || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!acc_fits(K, bits_x, bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < fwd_q_workspace_bytes(K, N)) return AQT_ERR_WORKSPACE;
  return launch_dense_fwd_q(xq, s_x, wq_packed, s_w, M, K, N, bits_w, bias, epilogue, y, acc_out, nullptr, ws,
                            static_cast<hipStream_t>(stream));
}

aqt_status aqt_dense_fwd_q_static(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                                  int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                                  int epilogue, float *y, void *stream) {
  if (!xq || !s_x || !wq_packed || !s_w || !y || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!acc_fits(K, bits_x, bits_w)) return AQT_ERR_UNSUPPORTED;
  if (K > static_cast<int64_t>(AQT_STATIC_SCRATCH_BYTES) / N ||
      fwd_q_workspace_bytes(K, N) > static_cast<size_t>(AQT_STATIC_SCRATCH_BYTES))
    return AQT_ERR_SCRATCH;
  void *ws = nullptr;
  AQT_TRY(static_scratch_address(&ws));
  return launch_dense_fwd_q(xq, s_x, wq_packed, s_w, M, K, N, bits_w, bias, epilogue, y, nullptr, nullptr, ws,
                            static_cast<hipStream_t>(stream));
}

size_t aqt_static_scratch_bytes(void) { return AQT_STATIC_SCRATCH_BYTES; }

size_t aqt_prepared_weight_bytes(int64_t K, int64_t N, int bits_w) {
  if (!shape_ok(K, N) || !bits_ok(bits_w) || K % 128 != 0 || N % 128 != 0) return 0;
  return static_cast<size_t>(K) * N / (packed4(bits_w) ? 2 : 1);
}

aqt_status aqt_prepare_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, void *wprep, void *stream) {
  if (!wq_packed || !wprep || !shape_ok(K, N)) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (K % 128 != 0 || N % 128 != 0) return AQT_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(wq_packed) % 16 != 0 || reinterpret_cast<uintptr_t>(wprep) % 16 != 0)
    return AQT_ERR_INVALID_ARG;
  return launch_prepare_weights(wq_packed, K, N, bits_w, wprep, static_cast<hipStream_t>(stream));
}

aqt_status aqt_dense_fwd_q_prepared(const int8_t *xq, const float *s_x, const void *wprep, const float *s_w,
                                    int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                                    int epilogue, float *y, void *stream) {
  if (!xq || !s_x || !wprep || !s_w || !y || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!acc_fits(K, bits_x, bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!fwd_q_takes_fragments(M, K, N, epilogue)) return AQT_ERR_UNSUPPORTED;
  if (reinterpret_cast<uintptr_t>(xq) % 16 != 0 || reinterpret_cast<uintptr_t>(wprep) % 16 != 0)
    return AQT_ERR_INVALID_ARG;
  return launch_dense_fwd_q(xq, s_x, nullptr, s_w, M, K, N, bits_w, bias, epilogue, y, nullptr, nullptr,
                            const_cast<void *>(wprep), static_cast<hipStream_t>(stream), nullptr, true);
}

aqt_status aqt_dense_fwd_q_absmax(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                                  int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                                  int epilogue, float *y, float *y_absmax, void *ws, size_t ws_bytes,
                                  void *stream) {
  if (!xq || !s_x || !wq_packed || !s_w || !y || !y_absmax || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!acc_fits(K, bits_x, bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < fwd_q_workspace_bytes(K, N)) return AQT_ERR_WORKSPACE;
  return launch_dense_fwd_q(xq, s_x, wq_packed, s_w, M, K, N, bits_w, bias, epilogue, y, nullptr,
                            reinterpret_cast<uint32_t *>(y_absmax), ws, static_cast<hipStream_t>(stream));
}

aqt_status aqt_dense_fwd_wonly(const float *x, const void *wq_packed, const float *s_w, int64_t M, int64_t K,
                               int64_t N, int bits_w, const float *bias, int epilogue, float *y, void *ws,
                               size_t ws_bytes, void *stream) {
  if (!x || !wq_packed || !s_w || !y || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < fwd_wonly_workspace_bytes(K, N)) return AQT_ERR_WORKSPACE;
  return launch_dense_fwd_wonly(x, wq_packed, s_w, M, K, N, bits_w, bias, epilogue, y, ws,
                                static_cast<hipStream_t>(stream));
}

aqt_status aqt_quantize_with_absmax(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                    const float *absmax, int8_t *q, float *scale, uint32_t *clip_mask,
                                    void *stream, int32_t *dev_status) {
  if (!x || !absmax || !q || !scale || !shape_ok(rows, cols) || ldx < cols) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits)) return AQT_ERR_UNSUPPORTED;
  return launch_quantize_with_absmax(x, rows, cols, ldx, bits, reinterpret_cast<const uint32_t *>(absmax), q, scale,
                                     clip_mask, static_cast<hipStream_t>(stream), dev_status);
}

aqt_status aqt_dense_fwd(const float *x, const float *w, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w,
                         const float *bias, int epilogue, float *y, const aqt_saved *saved, void *ws,
                         size_t ws_bytes, void *stream, int32_t *dev_status) {
  if (!x || !w || !y || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!acc_fits(K, bits_x, bits_w)) return AQT_ERR_UNSUPPORTED;
  FwdWorkspace f = carve_fwd(ws, M, K, N, bits_w);
  if (!ws || ws_bytes < f.total) return AQT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  int8_t *xq = (saved && saved->xq) ? saved->xq : f.xq;
  float *s_x = (saved && saved->s_x) ? saved->s_x : f.s_x;
  void *wq = (saved && saved->wq_packed) ? saved->wq_packed : f.wq;
  float *s_w = (saved && saved->s_w) ? saved->s_w : f.s_w;
  AQT_TRY(launch_quantize(x, M, K, K, bits_x, AQT_AXIS_ALL, xq, s_x, saved ? saved->mask_x : nullptr,
                          f.partials, st, dev_status));
  // when the matrix-core kernel takes the shape, the weight quantizer emits its operand in fragment order itself
  const bool frag = fwd_q_takes_fragments(M, K, N, epilogue) && reinterpret_cast<uintptr_t>(xq) % 16 == 0 &&
                    reinterpret_cast<uintptr_t>(f.wfrag) % 16 == 0;
  AQT_TRY(launch_quantize_weights(w, K, N, bits_w, wq, s_w, saved ? saved->wq_kn : nullptr,
                                  saved ? saved->mask_w : nullptr, f.wpart, st, dev_status, frag ? f.wfrag : nullptr));
  return launch_dense_fwd_q(xq, s_x, wq, s_w, M, K, N, bits_w, bias, epilogue, y, nullptr, nullptr, f.wfrag, st,
                            saved ? saved->dact : nullptr, frag);
}

aqt_status aqt_dense_bwd(const float *dy, const aqt_saved *saved, int64_t M, int64_t K, int64_t N, int bits_x,
                         int bits_w, int epilogue, float *dx, float *dw, float *dbias, void *ws, size_t ws_bytes,
                         void *stream) {
  if (!dy || !saved || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && epilogue != AQT_EPI_SWISH && epilogue != AQT_EPI_GLU) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (epilogue == AQT_EPI_GLU && (N % 2)) return AQT_ERR_UNSUPPORTED;
  if (!saved->s_x || !saved->s_w) return AQT_ERR_INVALID_ARG;
  if (dx && !saved->wq_kn) return AQT_ERR_INVALID_ARG;
  if (dw && !saved->xq) return AQT_ERR_INVALID_ARG;
  if (epilogue != AQT_EPI_NONE && !saved->dact) return AQT_ERR_INVALID_ARG;
  const size_t core = bwd_workspace_bytes(M, K, N);
  const size_t need = core + (epilogue != AQT_EPI_NONE ? align_up(static_cast<size_t>(M) * N * sizeof(float), 256) : 0);
  if (!ws || ws_bytes < need) return AQT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const float *dv = dy;
  if (epilogue != AQT_EPI_NONE) {
    // chain rule through the activation first: dv = dy * dact, [M,N], behind the core workspace
    float *buf = reinterpret_cast<float *>(static_cast<uint8_t *>(ws) + core);
    AQT_TRY(launch_dact_mul(dy, saved->dact, M, N, epilogue == AQT_EPI_GLU ? N / 2 : N, buf, st));
    dv = buf;
  }
  return launch_dense_bwd(dv, saved, M, K, N, dx, dw, dbias, ws, core, st);
}

aqt_status aqt_layernorm_quantize(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                                  float eps, int bits, int8_t *q, float *scale, float *y_out, float *row_stats,
                                  void *ws, size_t ws_bytes, void *stream, int32_t *dev_status) {
  if (!x || !shape_ok(M, D) || !(eps >= 0.0f)) return AQT_ERR_INVALID_ARG;
  if ((q == nullptr) != (scale == nullptr)) return AQT_ERR_INVALID_ARG;
  if (!q && !y_out) return AQT_ERR_INVALID_ARG;
  if (q && !bits_ok(bits)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < layernorm_ws_bytes(M)) return AQT_ERR_WORKSPACE;
  return launch_layernorm_quantize(x, M, D, gamma, beta, eps, bits, q, scale, y_out, row_stats, ws,
                                   static_cast<hipStream_t>(stream), dev_status);
}

aqt_status aqt_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N, float *out,
                               void *stream) {
  if (!xq || !wq_kn || !out || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (M >= (int64_t(1) << 31) / (K > N ? K : N) || cdiv(M, 128) > 65535) return AQT_ERR_UNSUPPORTED;
  return launch_fake_matmul_f32(xq, wq_kn, M, K, N, out, static_cast<hipStream_t>(stream));
}

aqt_status aqt_policy_preset(int pattern, int n_layers, int k, int bits_w, int bits_x, aqt_layer_policy *out) {
  if (!out || n_layers < 1) return AQT_ERR_INVALID_ARG;
  if (pattern < AQT_POLICY_ALL || pattern > AQT_POLICY_FIRST_K) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_w) || !(bits_x == 0 || bits_ok(bits_x))) return AQT_ERR_UNSUPPORTED;
  if (pattern == AQT_POLICY_FIRST_K && (k < 0 || k > n_layers)) return AQT_ERR_INVALID_ARG;
  const aqt_dense_policy low = {bits_w, bits_x, 0}, base = {8, bits_x, 0};   // Table 2: int8 for what is not selected
  for (int l = 0; l < n_layers; ++l) {
    bool sel = true;
    if (pattern == AQT_POLICY_EXCEPT_FIRST_LAST) sel = (l != 0 && l != n_layers - 1);
    if (pattern == AQT_POLICY_FIRST_K) sel = (l < k);
    const aqt_dense_policy p = sel ? low : base;
    aqt_layer_policy &o = out[l];
    o.ffn1_in = o.ffn1_out = o.conv_pw1 = o.conv_pw2 = o.ffn2_in = o.ffn2_out = p;
    o.attn_qkv = o.attn_out = (pattern == AQT_POLICY_EXCEPT_ATTENTION) ? base : p;
  }
  return AQT_OK;
}

size_t aqt_policy_weight_bytes(const aqt_layer_policy *policy, int n_layers, int64_t d_model, int64_t d_ff) {
  if (!policy || n_layers < 1 || d_model < 1 || d_ff < 1) return 0;
  size_t total = 0;
  auto add = [&](const aqt_dense_policy &p, int64_t K, int64_t N) {
    total += aqt_packed_weight_bytes(K, N, p.bits_w) + static_cast<size_t>(N) * sizeof(float);
  };
  for (int l = 0; l < n_layers; ++l) {
    const aqt_layer_policy &p = policy[l];
    if (!policy_ok(p.ffn1_in) || !policy_ok(p.ffn1_out) || !policy_ok(p.attn_qkv) || !policy_ok(p.attn_out) ||
        !policy_ok(p.conv_pw1) || !policy_ok(p.conv_pw2) || !policy_ok(p.ffn2_in) || !policy_ok(p.ffn2_out))
      return 0;
    add(p.ffn1_in, d_model, d_ff);  add(p.ffn1_out, d_ff, d_model);
    add(p.attn_qkv, d_model, 3 * d_model);  add(p.attn_out, d_model, d_model);
    add(p.conv_pw1, d_model, 2 * d_model);  add(p.conv_pw2, d_model, d_model);
    add(p.ffn2_in, d_model, d_ff);  add(p.ffn2_out, d_ff, d_model);
  }
  return total;
}

aqt_status aqt_ffn_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps, const float *w1,
                       const float *b1, const float *w2, const float *b2, int64_t M, int64_t D, int64_t H,
                       const aqt_dense_policy *policy, float *y, const aqt_ffn_saved *saved, void *ws,
                       size_t ws_bytes, void *stream, int32_t *dev_status) {
  return ffn_fwd_impl(x, ln_gamma, ln_beta, ln_eps, w1, b1, w2, b2, M, D, H, policy, y, saved, ws, ws_bytes, stream, dev_status, nullptr);
}

aqt_status aqt_ffn_bwd(const float *dy, const aqt_ffn_saved *saved, int64_t M, int64_t D, int64_t H,
                       const aqt_dense_policy *policy, float *dxn, float *dw1, float *db1, float *dw2, float *db2,
                       void *ws, size_t ws_bytes, void *stream) {
  AQT_TRY(ffn_bwd_check(dy, saved, M, D, H, policy, dxn, dw1, dw2, ws, ws_bytes));
  const aqt_saved &l1 = saved->l1, &l2 = saved->l2;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t a = bwd_workspace_bytes(M, D, H), b = bwd_workspace_bytes(M, H, D);
  const size_t core = a > b ? a : b;
  float *dh = reinterpret_cast<float *>(static_cast<uint8_t *>(ws) + core);
  // second layer (no activation): dw2, db2 and the gradient with respect to h, which leaves the kernel already
  // multiplied by the Swish derivative the first layer's forward stored; then the first layer
  const bool more = dxn || dw1 || db1;
  AQT_TRY(launch_dense_bwd(dy, &l2, M, H, D, dh, dw2, db2, ws, core, st, more ? l1.dact : nullptr));
  if (!more) return AQT_OK;
  return launch_dense_bwd(dh, &l1, M, D, H, dxn, dw1, db1, ws, core, st);
}

aqt_status aqt_depthwise_conv_fwd(const float *x, int64_t B, int64_t T, int64_t C, const float *w, const float *bias,
                                  int kw, int pad_left, const float *norm_scale, const float *norm_shift, int swish,
                                  float *out, float *dfac, float *out_absmax, void *stream) {
  if (!x || !w || !out || !conv_shape_ok(B, T, C, kw, pad_left)) return AQT_ERR_INVALID_ARG;
  return launch_dwconv_fwd(x, w, bias, norm_scale, norm_shift, swish ? 1 : 0, B, T, C, kw, pad_left, out, dfac,
                           reinterpret_cast<uint32_t *>(out_absmax), static_cast<hipStream_t>(stream));
}

aqt_status aqt_depthwise_conv_bwd(const float *dout, const float *dfac, const float *x, const float *w, int64_t B,
                                  int64_t T, int64_t C, int kw, int pad_left, float *dx, float *dw, float *dbias,
                                  void *ws, size_t ws_bytes, void *stream) {
  if (!dout || !conv_shape_ok(B, T, C, kw, pad_left)) return AQT_ERR_INVALID_ARG;
  if ((dx && !w) || (dw && !x)) return AQT_ERR_INVALID_ARG;
  if ((dw || dbias) && (!ws || ws_bytes < dwconv_bwd_ws_bytes(C, kw))) return AQT_ERR_WORKSPACE;
  // the bias sum rides with the tap sums and reads x only for the taps; give it a valid pointer
  return launch_dwconv_bwd(dout, dfac, x ? x : dout, w, B, T, C, kw, pad_left, dx, dw, dbias, ws,
                           static_cast<hipStream_t>(stream));
}

aqt_status aqt_conv_module_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps,
                               const float *w1, const float *b1, const float *w_dw, const float *b_dw,
                               const float *norm_scale, const float *norm_shift, const float *w2, const float *b2,
                               int64_t B, int64_t T, int64_t D, int kw, int pad_left, const aqt_dense_policy *policy,
                               float *y, const aqt_conv_saved *saved, void *ws, size_t ws_bytes, void *stream,
                               int32_t *dev_status) {
  return conv_module_fwd_impl(x, ln_gamma, ln_beta, ln_eps, w1, b1, w_dw, b_dw, norm_scale, norm_shift, w2, b2, B, T, D, kw, pad_left, policy, y, saved, ws, ws_bytes, stream, dev_status, nullptr);
}

aqt_status aqt_conv_module_bwd(const float *dy, const aqt_conv_saved *saved, const float *w_dw, int64_t B, int64_t T,
                               int64_t D, int kw, int pad_left, const aqt_dense_policy *policy, float *dxn,
                               float *dw1, float *db1, float *dw_dw, float *db_dw, float *dw2, float *db2, void *ws,
                               size_t ws_bytes, void *stream) {
  AQT_TRY(conv_module_bwd_check(dy, saved, w_dw, B, T, D, kw, pad_left, policy, dxn, dw1, dw2, ws, ws_bytes));
  const aqt_saved &l1 = saved->pw1, &l2 = saved->pw2;
  const int64_t M = B * T;
  ConvBwdWorkspace f = carve_conv_bwd(ws, B, T, D, kw);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // second pointwise convolution: gradient with respect to s, dw2, db2
  AQT_TRY(launch_dense_bwd(dy, &l2, M, D, D, f.ds, dw2, db2, ws, f.core, st));
  // through Swish and normalisation (dfac), then the depthwise convolution
  const bool more = dxn || dw1 || db1;
  AQT_TRY(launch_dwconv_bwd(f.ds, saved->dfac, saved->g, w_dw, B, T, D, kw, pad_left, more ? f.dg : nullptr, dw_dw,
                            db_dw, f.taps, st));
  if (!more) return AQT_OK;
  // through the GLU, then the first pointwise convolution
  AQT_TRY(launch_dact_mul(f.dg, l1.dact, M, 2 * D, D, f.dv, st));
  return launch_dense_bwd(f.dv, &l1, M, D, 2 * D, dxn, dw1, db1, ws, f.core, st);
}

aqt_status aqt_attention_fwd(const float *qkv, int64_t B, int64_t T, int64_t D, int heads, int left_context,
                             int right_context, float *ctx, float *ctx_absmax, float *lse, void *stream) {
  if (!qkv || !ctx || B < 1 || T < 1 || D < 1 || heads < 1 || D % heads) return AQT_ERR_INVALID_ARG;
  if (!attention_shape_ok(B, T, D, heads)) return AQT_ERR_UNSUPPORTED;
  return launch_attention(qkv, B, T, D, heads, left_context, right_context, ctx,
                          reinterpret_cast<uint32_t *>(ctx_absmax), lse, static_cast<hipStream_t>(stream));
}

aqt_status aqt_attention_bwd(const float *qkv, const float *ctx, const float *dctx, const float *lse, int64_t B,
                             int64_t T, int64_t D, int heads, int left_context, int right_context, float *dqkv,
                             void *ws, size_t ws_bytes, void *stream) {
  if (!qkv || !ctx || !dctx || !lse || !dqkv || B < 1 || T < 1 || D < 1 || heads < 1 || D % heads)
    return AQT_ERR_INVALID_ARG;
  if (!attention_shape_ok(B, T, D, heads)) return AQT_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < attention_bwd_ws_bytes(B, T, heads)) return AQT_ERR_WORKSPACE;
  return launch_attention_bwd(qkv, ctx, dctx, lse, B, T, D, heads, left_context, right_context, dqkv, ws,
                              static_cast<hipStream_t>(stream));
}

aqt_status aqt_mhsa_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps, const float *wqkv,
                        const float *bqkv, const float *wo, const float *bo, int64_t B, int64_t T, int64_t D,
                        int heads, int left_context, int right_context, const aqt_dense_policy *policy, float *y,
                        const aqt_mhsa_saved *saved, void *ws, size_t ws_bytes, void *stream, int32_t *dev_status) {
  return mhsa_fwd_impl(x, ln_gamma, ln_beta, ln_eps, wqkv, bqkv, wo, bo, B, T, D, heads, left_context, right_context, policy, y, saved, ws, ws_bytes, stream, dev_status, nullptr);
}

aqt_status aqt_residual_add(const float *x, const float *m, float alpha, float *out, int64_t n, void *stream) {
  if (!x || !m || !out || n < 1) return AQT_ERR_INVALID_ARG;
  return launch_residual_add(x, m, alpha, out, n, static_cast<hipStream_t>(stream));
}

aqt_status aqt_conformer_layer_fwd(const float *x, const aqt_conformer_layer_weights *w,
                                   const aqt_conformer_layer_shape *shape, const aqt_layer_policy *policy, float *y,
                                   const aqt_conformer_layer_saved *saved, void *ws, size_t ws_bytes, void *stream,
                                   int32_t *dev_status) {
  if (!x || !w || !shape || !policy || !y || !saved) return AQT_ERR_INVALID_ARG;
  const aqt_conformer_layer_shape &g = *shape;
  if (g.B < 1 || g.T < 1 || g.D < 1 || g.H < 1 || g.B > (int64_t(1) << 40) / g.T) return AQT_ERR_INVALID_ARG;
  if (!saved->r1 || !saved->r2 || !saved->r3 || !saved->r4 || !saved->m) return AQT_ERR_INVALID_ARG;
  const int64_t M = g.B * g.T;
  if (!ws || ws_bytes < aqt_workspace_bytes(AQT_OP_CONFORMER_LAYER_FWD, M, g.D, g.H, 8, 8)) return AQT_ERR_WORKSPACE;
  const aqt_dense_policy pf1[2] = {policy->ffn1_in, policy->ffn1_out}, pa[2] = {policy->attn_qkv, policy->attn_out};
  const aqt_dense_policy pc[2] = {policy->conv_pw1, policy->conv_pw2}, pf2[2] = {policy->ffn2_in, policy->ffn2_out};
  // every module's own checks, before the first launch: a call that is going to be refused leaves no buffer half written
  AQT_TRY(ffn_fwd_check(x, g.ln_eps, w->ffn1_w1, w->ffn1_w2, M, g.D, g.H, pf1, saved->m, &saved->ffn1, ws, ws_bytes));
  AQT_TRY(mhsa_fwd_check(x, g.ln_eps, w->att_wqkv, w->att_wo, g.B, g.T, g.D, g.heads, pa, saved->m, &saved->att, ws,
                         ws_bytes));
  AQT_TRY(conv_module_fwd_check(saved->r1, g.ln_eps, w->conv_w1, w->conv_wdw, w->conv_w2, g.B, g.T, g.D, g.kw,
                                g.pad_left, pc, saved->m, &saved->conv, ws, ws_bytes));
  AQT_TRY(ffn_fwd_check(saved->r2, g.ln_eps, w->ffn2_w1, w->ffn2_w2, M, g.D, g.H, pf2, saved->m, &saved->ffn2, ws,
                        ws_bytes));
  // every weight matrix of the layer that is not already in serving form goes through the weight quantizer in one
  // launch pair; the modules then find their weight side ready
  hipStream_t st = static_cast<hipStream_t>(stream);
  const LayerFwdWorkspace lw = carve_layer_fwd(ws, M, g.D, g.H);
  WeightJobList jobs;
  WeightSide sd[8];
  const int64_t D = g.D, H = g.H;
  AQT_TRY(weight_side(pf1[0], w->ffn1_w1, saved->ffn1.l1, M, D, H, AQT_EPI_SWISH, lw.wpart[0], lw.wfrag[0], st,
                      dev_status, &sd[0], &jobs));
  AQT_TRY(weight_side(pf1[1], w->ffn1_w2, saved->ffn1.l2, M, H, D, AQT_EPI_NONE, lw.wpart[1], lw.wfrag[1], st,
                      dev_status, &sd[1], &jobs));
  AQT_TRY(weight_side(pa[0], w->att_wqkv, saved->att.qkv, M, D, 3 * D, AQT_EPI_NONE, lw.wpart[2], lw.wfrag[2], st,
                      dev_status, &sd[2], &jobs));
  AQT_TRY(weight_side(pa[1], w->att_wo, saved->att.out, M, D, D, AQT_EPI_NONE, lw.wpart[3], lw.wfrag[3], st,
                      dev_status, &sd[3], &jobs));
  AQT_TRY(weight_side(pc[0], w->conv_w1, saved->conv.pw1, M, D, 2 * D, AQT_EPI_GLU, lw.wpart[4], lw.wfrag[4], st,
                      dev_status, &sd[4], &jobs));
  AQT_TRY(weight_side(pc[1], w->conv_w2, saved->conv.pw2, M, D, D, AQT_EPI_NONE, lw.wpart[5], lw.wfrag[5], st,
                      dev_status, &sd[5], &jobs));
  AQT_TRY(weight_side(pf2[0], w->ffn2_w1, saved->ffn2.l1, M, D, H, AQT_EPI_SWISH, lw.wpart[6], lw.wfrag[6], st,
                      dev_status, &sd[6], &jobs));
  AQT_TRY(weight_side(pf2[1], w->ffn2_w2, saved->ffn2.l2, M, H, D, AQT_EPI_NONE, lw.wpart[7], lw.wfrag[7], st,
                      dev_status, &sd[7], &jobs));
  AQT_TRY(launch_quantize_weights_group(jobs.job, jobs.n, st, dev_status));
  // half-step feed-forward module.  From here on the residual connection in front of a module is formed by that
  // module's normalisation pass: r = r_prev + alpha * (previous module's output), left in saved->r*.
  AQT_TRY(ffn_fwd_impl(x, w->ffn1_ln_g, w->ffn1_ln_b, g.ln_eps, w->ffn1_w1, w->ffn1_b1, w->ffn1_w2, w->ffn1_b2, M, g.D,
                       g.H, pf1, saved->m, &saved->ffn1, ws, lw.module, stream, dev_status, nullptr, &sd[0]));
  // self-attention module on r1 = x + ffn(x) / 2
  const ResidualIn in1 = {saved->m, 0.5f, saved->r1};
  AQT_TRY(mhsa_fwd_impl(x, w->att_ln_g, w->att_ln_b, g.ln_eps, w->att_wqkv, w->att_bqkv, w->att_wo, w->att_bo, g.B, g.T,
                        g.D, g.heads, g.left_context, g.right_context, pa, saved->m, &saved->att, ws, lw.module, stream,
                        dev_status, &in1, &sd[2]));
  // convolution module on r2 = r1 + mhsa(r1)
  const ResidualIn in2 = {saved->m, 1.0f, saved->r2};
  AQT_TRY(conv_module_fwd_impl(saved->r1, w->conv_ln_g, w->conv_ln_b, g.ln_eps, w->conv_w1, w->conv_b1, w->conv_wdw,
                               w->conv_bdw, w->conv_norm_scale, w->conv_norm_shift, w->conv_w2, w->conv_b2, g.B, g.T,
                               g.D, g.kw, g.pad_left, pc, saved->m, &saved->conv, ws, lw.module, stream, dev_status,
                               &in2, &sd[4]));
  // second half-step feed-forward module on r3 = r2 + conv(r2)
  const ResidualIn in3 = {saved->m, 1.0f, saved->r3};
  AQT_TRY(ffn_fwd_impl(saved->r2, w->ffn2_ln_g, w->ffn2_ln_b, g.ln_eps, w->ffn2_w1, w->ffn2_b1, w->ffn2_w2, w->ffn2_b2,
                       M, g.D, g.H, pf2, saved->m, &saved->ffn2, ws, lw.module, stream, dev_status, &in3, &sd[6]));
  // final normalisation of r4 = r3 + ffn(r3) / 2
  return launch_layernorm_quantize(saved->r3, M, g.D, w->out_ln_g, w->out_ln_b, g.ln_eps, 8, nullptr, nullptr, y,
                                   saved->out_row_stats, ws, static_cast<hipStream_t>(stream), dev_status, saved->m,
                                   0.5f, saved->r4);
}

aqt_status aqt_layernorm_bwd(const float *x, const float *row_stats, const float *gamma, const float *dy,
                             const float *add, int64_t M, int64_t D, float *dx, float *dgamma, float *dbeta,
                             void *ws, size_t ws_bytes, void *stream) {
  if (!x || !row_stats || !dy || !dx || !shape_ok(M, D)) return AQT_ERR_INVALID_ARG;
  if ((dgamma || dbeta) && (!ws || ws_bytes < layernorm_bwd_ws_bytes(D))) return AQT_ERR_WORKSPACE;
  return launch_layernorm_bwd(x, row_stats, gamma, dy, add, M, D, dx, dgamma, dbeta, ws,
                              static_cast<hipStream_t>(stream));
}

aqt_status aqt_mhsa_bwd(const float *dy, const aqt_mhsa_saved *saved, int64_t B, int64_t T, int64_t D, int heads,
                        int left_context, int right_context, const aqt_dense_policy *policy, float *dxn,
                        float *dwqkv, float *dbqkv, float *dwo, float *dbo, void *ws, size_t ws_bytes, void *stream) {
  AQT_TRY(mhsa_bwd_check(dy, saved, B, T, D, heads, policy, dxn, dwqkv, dwo, ws, ws_bytes));
  const aqt_saved &l1 = saved->qkv, &l2 = saved->out;
  const int64_t M = B * T;
  MhsaBwdWorkspace f = carve_mhsa_bwd(ws, M, D, heads);
  hipStream_t st = static_cast<hipStream_t>(stream);
  // output projection: gradient with respect to the attention result
  AQT_TRY(launch_dense_bwd(dy, &l2, M, D, D, f.dctx, dwo, dbo, ws, f.core, st));
  if (!dxn && !dwqkv && !dbqkv) return AQT_OK;
  // attention, then the fused projection
  AQT_TRY(launch_attention_bwd(saved->qkv_f, saved->ctx, f.dctx, saved->lse, B, T, D, heads, left_context,
                               right_context, f.dqkv, f.att, st));
  return launch_dense_bwd(f.dqkv, &l1, M, D, 3 * D, dxn, dwqkv, dbqkv, ws, f.core, st);
}

aqt_status aqt_conformer_layer_bwd(const float *dy, const float *x, const aqt_conformer_layer_weights *w,
                                   const aqt_conformer_layer_shape *shape, const aqt_layer_policy *policy,
                                   const aqt_conformer_layer_saved *saved, float *dx,
                                   const aqt_conformer_layer_grads *grads, void *ws, size_t ws_bytes, void *stream) {
  if (!dy || !x || !w || !shape || !policy || !saved || !dx || !grads) return AQT_ERR_INVALID_ARG;
  const aqt_conformer_layer_shape &g = *shape;
  if (g.B < 1 || g.T < 1 || g.D < 1 || g.H < 1 || g.B > (int64_t(1) << 40) / g.T) return AQT_ERR_INVALID_ARG;
  if (grads->conv_norm_scale || grads->conv_norm_shift) return AQT_ERR_UNSUPPORTED;
  if (!saved->r1 || !saved->r2 || !saved->r3 || !saved->r4 || !saved->out_row_stats || !saved->ffn1.row_stats ||
      !saved->ffn2.row_stats || !saved->att.row_stats || !saved->conv.row_stats || !w->conv_wdw)
    return AQT_ERR_INVALID_ARG;
  if (!conv_shape_ok(g.B, g.T, g.D, g.kw, g.pad_left) || !attention_shape_ok(g.B, g.T, g.D, g.heads))
    return AQT_ERR_UNSUPPORTED;
  const int64_t M = g.B * g.T, n = M * g.D;
  LayerBwdWorkspace f = carve_layer_bwd(ws, M, g.D, g.H, g.heads, g.kw);
  if (!ws || ws_bytes < f.total) return AQT_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const aqt_dense_policy pf1[2] = {policy->ffn1_in, policy->ffn1_out}, pa[2] = {policy->attn_qkv, policy->attn_out};
  const aqt_dense_policy pc[2] = {policy->conv_pw1, policy->conv_pw2}, pf2[2] = {policy->ffn2_in, policy->ffn2_out};
  // the modules' own checks, before the first launch (f.dm, f.da, f.db stand for the gradients they will be given)
  AQT_TRY(ffn_bwd_check(f.dm, &saved->ffn2, M, g.D, g.H, pf2, f.dm, grads->ffn2_w1, grads->ffn2_w2, ws, f.module));
  AQT_TRY(conv_module_bwd_check(f.db, &saved->conv, w->conv_wdw, g.B, g.T, g.D, g.kw, g.pad_left, pc, f.dm,
                                grads->conv_w1, grads->conv_w2, ws, f.module));
  AQT_TRY(mhsa_bwd_check(f.da, &saved->att, g.B, g.T, g.D, g.heads, pa, f.dm, grads->att_wqkv, grads->att_wo, ws,
                         f.module));
  AQT_TRY(ffn_bwd_check(f.dm, &saved->ffn1, M, g.D, g.H, pf1, f.dm, grads->ffn1_w1, grads->ffn1_w2, ws, f.module));
  // final normalisation: gradient of the residual stream r4
  AQT_TRY(launch_layernorm_bwd(saved->r4, saved->out_row_stats, w->out_ln_g, dy, nullptr, M, g.D, f.da, grads->out_ln_g,
                               grads->out_ln_b, f.ln, st));
  // second feed-forward module entered the stream with weight 1/2: r4 = r3 + ffn(r3) / 2
  AQT_TRY(launch_scale(f.da, 0.5f, f.dm, n, st));
  AQT_TRY(aqt_ffn_bwd(f.dm, &saved->ffn2, M, g.D, g.H, pf2, f.dm, grads->ffn2_w1, grads->ffn2_b1, grads->ffn2_w2,
                      grads->ffn2_b2, ws, f.module, stream));
  AQT_TRY(launch_layernorm_bwd(saved->r3, saved->ffn2.row_stats, w->ffn2_ln_g, f.dm, f.da, M, g.D, f.db,
                               grads->ffn2_ln_g, grads->ffn2_ln_b, f.ln, st));
  // convolution module: r3 = r2 + conv(r2)
  AQT_TRY(aqt_conv_module_bwd(f.db, &saved->conv, w->conv_wdw, g.B, g.T, g.D, g.kw, g.pad_left, pc, f.dm,
                              grads->conv_w1, grads->conv_b1, grads->conv_wdw, grads->conv_bdw, grads->conv_w2,
                              grads->conv_b2, ws, f.module, stream));
  AQT_TRY(launch_layernorm_bwd(saved->r2, saved->conv.row_stats, w->conv_ln_g, f.dm, f.db, M, g.D, f.da,
                               grads->conv_ln_g, grads->conv_ln_b, f.ln, st));
  // self-attention module: r2 = r1 + mhsa(r1)
  AQT_TRY(aqt_mhsa_bwd(f.da, &saved->att, g.B, g.T, g.D, g.heads, g.left_context, g.right_context, pa, f.dm,
                       grads->att_wqkv, grads->att_bqkv, grads->att_wo, grads->att_bo, ws, f.module, stream));
  AQT_TRY(launch_layernorm_bwd(saved->r1, saved->att.row_stats, w->att_ln_g, f.dm, f.da, M, g.D, f.db,
                               grads->att_ln_g, grads->att_ln_b, f.ln, st));
  // first feed-forward module: r1 = x + ffn(x) / 2
  AQT_TRY(launch_scale(f.db, 0.5f, f.dm, n, st));
  AQT_TRY(aqt_ffn_bwd(f.dm, &saved->ffn1, M, g.D, g.H, pf1, f.dm, grads->ffn1_w1, grads->ffn1_b1, grads->ffn1_w2,
                      grads->ffn1_b2, ws, f.module, stream));
  return launch_layernorm_bwd(x, saved->ffn1.row_stats, w->ffn1_ln_g, f.dm, f.db, M, g.D, dx, grads->ffn1_ln_g,
                              grads->ffn1_ln_b, f.ln, st);
}

}  // extern "C"
