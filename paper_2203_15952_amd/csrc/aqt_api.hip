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

// The int32 accumulator must hold K * qmax_x * qmax_w; packed (<= 4 bit) weights enter the
// matrix cores as 16 * code, so their sums carry a factor 16 until the final shift.
bool acc_fits(int64_t K, int bits_x, int bits_w) {
  const int64_t lim = (int64_t(1) << 31) / (packed4(bits_w) ? 16 : 1);
  return K * qmax_of(bits_x) * qmax_of(bits_w) < lim;
}

}  // namespace
}  // namespace aqt

using namespace aqt;

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

int aqt_version(void) { return 100; }

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
  AQT_TRY(launch_quantize_weights(w, K, N, bits_w, wq, s_w, saved ? saved->wq_kn : nullptr,
                                  saved ? saved->mask_w : nullptr, f.wpart, st, dev_status));
  return launch_dense_fwd_q(xq, s_x, wq, s_w, M, K, N, bits_w, bias, epilogue, y, nullptr, nullptr, f.wfrag, st);
}

aqt_status aqt_dense_bwd(const float *dy, const aqt_saved *saved, int64_t M, int64_t K, int64_t N, int bits_x,
                         int bits_w, float *dx, float *dw, float *dbias, void *ws, size_t ws_bytes,
                         void *stream) {
  if (!dy || !saved || !shape_ok(M, K) || N < 1) return AQT_ERR_INVALID_ARG;
  if (!bits_ok(bits_x) || !bits_ok(bits_w)) return AQT_ERR_UNSUPPORTED;
  if (!saved->s_x || !saved->s_w) return AQT_ERR_INVALID_ARG;
  if (dx && !saved->wq_kn) return AQT_ERR_INVALID_ARG;
  if (dw && !saved->xq) return AQT_ERR_INVALID_ARG;
  const size_t need = bwd_workspace_bytes(M, K, N);
  if (!ws || ws_bytes < need) return AQT_ERR_WORKSPACE;
  return launch_dense_bwd(dy, saved, M, K, N, dx, dw, dbias, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

}  // extern "C"
