// Internal declarations shared by the HIP translation units of libaqt.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aqt.h"

// Per-tile timelines (tracing builds only, -DAQT_TIMELINE; see paper_2203_15952_amd/timeline.py):
// wavefront 0 of every workgroup stamps the shader clock at its phase boundaries and leaves
// eight 64-bit words per workgroup in a device array of the translation unit, which an
// extern "C" accessor copies out.  The product build contains none of this.
#ifdef AQT_TIMELINE
#define AQT_TL_SLOTS (1 << 15)
#define AQT_TL_DECL long long aqt_tl_[5] = {0, 0, 0, 0, 0}
#define AQT_TL(i) aqt_tl_[i] = __builtin_readcyclecounter()
#define AQT_TL_WRITE(buf, tag)                                                        \
  do {                                                                                \
    if ((threadIdx.x & 63) == 0 && (threadIdx.x >> 6) == 0 && blockIdx.x < AQT_TL_SLOTS) { \
      unsigned hw_, xcc_;                                                             \
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw_));               \
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc_));             \
      long long *o_ = (buf) + static_cast<long long>(blockIdx.x) * 8;                 \
      o_[0] = aqt_tl_[0]; o_[1] = aqt_tl_[1]; o_[2] = aqt_tl_[2]; o_[3] = aqt_tl_[3];  \
      o_[4] = aqt_tl_[4]; o_[5] = hw_; o_[6] = xcc_; o_[7] = (tag);                    \
    }                                                                                 \
  } while (0)
#else
#define AQT_TL_DECL
#define AQT_TL(i)
#define AQT_TL_WRITE(buf, tag)
#endif

namespace aqt {

extern thread_local int g_last_hip_error;

#define AQT_HIP(expr)                                   \
  do {                                                  \
    hipError_t e__ = (expr);                            \
    if (e__ != hipSuccess) {                            \
      aqt::g_last_hip_error = static_cast<int>(e__);    \
      return AQT_ERR_HIP;                               \
    }                                                   \
  } while (0)

#define AQT_TRY(expr)                 \
  do {                                \
    aqt_status s__ = (expr);          \
    if (s__ != AQT_OK) return s__;    \
  } while (0)

constexpr int kMaxPartials = 4096;  // per-block abs-max slots at the head of a quantize workspace
constexpr int kWeightSlabs = 16;    // fan-in slabs whose per-channel maxima the weight quantizer folds

inline int qmax_of(int bits) { return (1 << (bits - 1)) - 1; }
inline bool bits_ok(int bits) { return bits >= 2 && bits <= 8; }
inline bool packed4(int bits_w) { return bits_w <= 4; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ __device__ inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- quantizers (quantize.hip) ------------------------------------------------
aqt_status launch_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int axis,
                           int8_t *q, float *scale, uint32_t *mask, float *partials, hipStream_t st,
                           int32_t *dev_status);
aqt_status launch_quantize_with_absmax(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                       const uint32_t *absmax_bits, int8_t *q, float *scale, uint32_t *mask,
                                       hipStream_t st, int32_t *dev_status);
aqt_status launch_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                      int axis, const float *scale, int8_t *q, uint32_t *mask,
                                      hipStream_t st);
aqt_status launch_quantize_weights(const float *w, int64_t K, int64_t N, int bits_w, void *wq_packed,
                                   float *s_w, int8_t *wq_kn, uint32_t *mask_w, uint32_t *part,
                                   hipStream_t st, int32_t *dev_status, void *wfrag = nullptr);
// Several matrices through the weight quantizer in one launch pair (same arithmetic per matrix).
struct WeightJob {
  const float *w;
  int64_t K, N;
  int bits_w;
  void *wq_packed;
  float *s_w;
  int8_t *wq_kn;       // nullable
  uint32_t *mask_w;    // nullable
  uint32_t *part;      // kWeightSlabs x N words of its own
  void *wfrag;         // nullable
};
constexpr int kWeightJobsMax = 8;
aqt_status launch_quantize_weights_group(const WeightJob *jobs, int n, hipStream_t st, int32_t *dev_status);
inline size_t weight_ws_bytes(int64_t N) { return align_up(static_cast<size_t>(kWeightSlabs) * N * 4, 256); }
aqt_status launch_unpack_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w,
                                 int8_t *codes_kn, hipStream_t st);

// ---- forward contraction (gemm_fwd.hip) -----------------------------------------
aqt_status launch_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed,
                              const float *s_w, int64_t M, int64_t K, int64_t N, int bits_w,
                              const float *bias, int epilogue, float *y, int32_t *acc_out, uint32_t *y_absmax,
                              void *ws, hipStream_t st, float *dact = nullptr, bool ws_is_prepared = false,
                              bool absmax_is_zero = false);
// True when the matrix-core kernel takes the shape (then its weight operand may be handed over
// already in fragment order: from the weight quantizer, or from launch_prepare_weights).
bool fwd_q_takes_fragments(int64_t M, int64_t K, int64_t N, int epilogue);
aqt_status launch_prepare_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, void *wprep,
                                  hipStream_t st);
size_t fwd_q_workspace_bytes(int64_t K, int64_t N);
aqt_status static_scratch_address(void **out);   // the library's own scratch array on the current device
size_t fwd_wonly_workspace_bytes(int64_t K, int64_t N);
aqt_status launch_dense_fwd_wonly(const float *x, const void *wq_packed, const float *s_w, int64_t M, int64_t K,
                                  int64_t N, int bits_w, const float *bias, int epilogue, float *y, void *ws,
                                  hipStream_t st);

// ---- straight-through backward (gemm_bwd.hip) -------------------------------------
size_t bwd_workspace_bytes(int64_t M, int64_t K, int64_t N);
// dx_factor (optional, [M,K]): dx leaves multiplied elementwise by it (the previous layer's activation derivative)
aqt_status launch_dense_bwd(const float *dy, const aqt_saved *sv, int64_t M, int64_t K, int64_t N,
                            float *dx, float *dw, float *dbias, void *ws, size_t ws_bytes,
                            hipStream_t st, const float *dx_factor = nullptr);

// ---- block pieces (block.hip) -----------------------------------------------------------
size_t layernorm_ws_bytes(int64_t M);
// res / alpha / sum_out (optional): normalise x + alpha * res instead of x and leave that sum in sum_out.
// zero_word (optional): a word the first pass clears, e.g. the abs-max word of a producer launched after it
// (which is then told absmax_is_zero and needs no clearing launch of its own).
aqt_status launch_layernorm_quantize(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                                     float eps, int bits, int8_t *q, float *scale, float *y_out, float *row_stats,
                                     void *ws, hipStream_t st, int32_t *dev_status, const float *res = nullptr,
                                     float alpha = 0.0f, float *sum_out = nullptr, uint32_t *zero_word = nullptr);
size_t layernorm_bwd_ws_bytes(int64_t D);
aqt_status launch_layernorm_bwd(const float *x, const float *stats, const float *gamma, const float *dy,
                                const float *add, int64_t M, int64_t D, float *dx, float *dgamma, float *dbeta,
                                void *ws, hipStream_t st);
aqt_status launch_scale(const float *m, float alpha, float *out, int64_t n, hipStream_t st);
aqt_status launch_dact_mul(const float *dout, const float *dact, int64_t M, int64_t N, int64_t oc, float *dv,
                           hipStream_t st);
aqt_status launch_residual_add(const float *x, const float *m, float alpha, float *out, int64_t n, hipStream_t st);
aqt_status launch_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N, float *out,
                                  hipStream_t st);

// ---- depthwise convolution of the convolution module (conv.hip) ---------------------------
size_t dwconv_bwd_ws_bytes(int64_t C, int kw);
aqt_status launch_dwconv_fwd(const float *x, const float *w, const float *bias, const float *na, const float *nb,
                             int swish, int64_t B, int64_t T, int64_t C, int kw, int pad_left, float *out, float *dfac,
                             uint32_t *absmax, hipStream_t st, bool absmax_is_zero = false);
aqt_status launch_dwconv_bwd(const float *dout, const float *dmul, const float *x, const float *w, int64_t B, int64_t T,
                             int64_t C, int kw, int pad_left, float *dx, float *dw, float *dbias, void *ws,
                             hipStream_t st);

// ---- attention core of the self-attention module (attention.hip) ---------------------------
bool attention_shape_ok(int64_t B, int64_t T, int64_t D, int heads);
aqt_status launch_attention(const float *qkv, int64_t B, int64_t T, int64_t D, int heads, int left, int right,
                            float *ctx, uint32_t *absmax, float *lse, hipStream_t st, bool absmax_is_zero = false);
size_t attention_bwd_ws_bytes(int64_t B, int64_t T, int heads);
aqt_status launch_attention_bwd(const float *qkv, const float *ctx, const float *dctx, const float *lse, int64_t B,
                                int64_t T, int64_t D, int heads, int left, int right, float *dqkv, void *ws,
                                hipStream_t st);

}  // namespace aqt
