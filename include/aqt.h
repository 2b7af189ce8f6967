/*
 * aqt.h -- C ABI of the MI355X (gfx950) quantized dense layer for native
 * quantization-aware training, arxiv 2203.15952 ("4-bit Conformer with Native
 * Quantization Aware Training for Speech Recognition").
 *
 * The layer (Sec. 1, Sec. 2.2, Fig. 2): activations are quantized symmetrically
 * per tensor and weights per output channel with abs-max scaling
 * (scale = max|v| / qmax, code = floor(v / scale + 0.5), qmax = 127 for int8 and
 * 7 for int4, no zero point), the product is taken in integers with an int32
 * accumulator, and the result is de-quantized by multiplying with the scales.
 * The backward pass treats the scales as constants (Fig. 2, stop_gradient) and
 * passes the rounding straight through.
 *
 * Conventions for every entry point
 *   - Pointers are DEVICE pointers unless a comment says "host"; the caller owns
 *     every buffer.  The library allocates and frees no device memory: scratch
 *     is a caller-supplied workspace (`ws`, `ws_bytes`), sized by
 *     aqt_workspace_bytes(), 256-byte aligned.  Calls that share a workspace
 *     must be ordered on one stream.
 *   - Tensors are dense row-major.  X is [M,K], W is [K,N] (K = fan-in, N =
 *     output channels), Y is [M,N].  Any M, K, N >= 1 is accepted; shapes that
 *     do not meet a tuned kernel's divisibility take a slower general kernel
 *     with identical results.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued and the call returns; argument errors are reported
 *     synchronously through the return value and enqueue nothing.
 *   - `dev_status` (nullable) is a device int32 the kernels set to
 *     AQT_ERR_NONFINITE when an abs-max is Inf/NaN.  The library never clears
 *     it; outputs are unspecified when it is set.
 *   - bits must lie in 2..8.  Codes always live in an int8 container; weights
 *     with bits_w <= 4 are additionally stored packed two per byte.
 */
#ifndef AQT_H
#define AQT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int aqt_status;
#define AQT_OK 0
#define AQT_ERR_INVALID_ARG 1 /* null pointer, non-positive size, bad axis/epilogue       */
#define AQT_ERR_UNSUPPORTED 2 /* bits outside 2..8, GLU with odd N, K too large for int32 */
#define AQT_ERR_WORKSPACE 3   /* ws is NULL or smaller than aqt_workspace_bytes()         */
#define AQT_ERR_HIP 4         /* a HIP call failed; see aqt_last_hip_error()              */
#define AQT_ERR_NONFINITE 5   /* only ever written to *dev_status by a kernel             */
#define AQT_ERR_SCRATCH 6     /* aqt_dense_fwd_q_static: K * N exceeds the static scratch */

/* `axis` names the REDUCED axes, as the `axis` argument of Fig. 2 does. */
#define AQT_AXIS_ALL (-1) /* one scale for the whole tensor (activations)              */
#define AQT_AXIS_ROWS 0   /* reduce over rows: one scale per column (W[K,N]: channel)  */
#define AQT_AXIS_COLS 1   /* reduce over columns: one scale per row                    */

#define AQT_EPI_NONE 0
#define AQT_EPI_SWISH 1 /* y * sigmoid(y)                                               */
#define AQT_EPI_GLU 2   /* y[:, j] * sigmoid(y[:, j + N/2]), j < N/2; output is [M,N/2] */

#define AQT_OP_QUANTIZE 0
#define AQT_OP_QUANTIZE_WEIGHTS 1
#define AQT_OP_DENSE_FWD 2
#define AQT_OP_DENSE_FWD_Q 3
#define AQT_OP_DENSE_BWD 4
#define AQT_OP_DENSE_FWD_WONLY 5

/* What the forward keeps for the backward.  All caller-owned device buffers. */
typedef struct aqt_saved {
  int8_t *xq;        /* [M,K] activation codes                                          */
  float *s_x;        /* [1]   activation scale                                          */
  uint32_t *mask_x;  /* nullable: ceil(M*K/32) words, bit i = element i, 1 = passes     */
  void *wq_packed;   /* forward operand, aqt_packed_weight_bytes(K,N,bits_w) bytes      */
  int8_t *wq_kn;     /* [K,N] weight codes in the layout of W (backward operand)        */
  float *s_w;        /* [N]   weight scales                                             */
  uint32_t *mask_w;  /* nullable: ceil(K*N/32) words over W's [K,N] order               */
} aqt_saved;

const char *aqt_status_string(aqt_status s); /* host, static storage */
int aqt_last_hip_error(void);                /* hipError_t of this thread's last failed HIP call */
int aqt_version(void);

/* Bytes of workspace an op needs for the given shape (host computation, no GPU). 0 on bad args. */
size_t aqt_workspace_bytes(int op, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w);

/*
 * Size of the forward weight operand.  Layout: N rows, fan-in contiguous.
 *   bits_w > 4 : int8  [N][K]
 *   bits_w <= 4: bytes [N][ceil(K/2)], byte j of a row holds k = 2j in its low
 *                nibble and k = 2j+1 in its high nibble, two's complement; an
 *                odd K leaves the last high nibble zero.  Code -8 never occurs.
 * Half a byte per int4 parameter is what the model sizes of Table 1 imply.
 */
size_t aqt_packed_weight_bytes(int64_t K, int64_t N, int bits_w);

/*
 * Fig. 2 with the bit-width rule of Sec. 2.2: per reduction group,
 * m = max|x|, scale = m / qmax, code = floor(x / scale + 0.5) (0 when scale is
 * 0), each operation one float32 rounding.
 *   x      [rows, cols] float32, row stride ldx (elements, >= cols)
 *   q      [rows, cols] int8 codes, dense
 *   scale  1, cols or rows float32 according to axis
 *   clip_mask  nullable, ceil(rows*cols/32) words, bit (i % 32) of word i/32 for
 *              element i = r*cols + c; 1 when the rounded value lies inside
 *              [-qmax, qmax] and the scale is non-zero (always, under abs-max
 *              scaling, for non-zero groups)
 */
aqt_status aqt_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int axis,
                        int8_t *q, float *scale, uint32_t *clip_mask, void *ws, size_t ws_bytes,
                        void *stream, int32_t *dev_status);

/*
 * The element-wise half of Fig. 2 with caller-supplied scales (device, 1 / cols
 * / rows floats according to axis): code = clamp(floor(x / scale + 0.5), -qmax,
 * qmax).  Only this form can saturate, so clip_mask (nullable, as above) is not
 * trivially all ones here.
 */
aqt_status aqt_quantize_with_scale(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                   int axis, const float *scale, int8_t *q, uint32_t *clip_mask,
                                   void *stream);

/*
 * Weights, Sec. 2.2 (channel-wise): quantize W[K,N] per output channel (reduce
 * over K) and emit the forward operand in the layout of
 * aqt_packed_weight_bytes().  wq_kn (nullable) also receives the codes as int8
 * in W's own [K,N] layout, which is what the backward contracts with;
 * clip_mask_w nullable, bit order of W[K,N].  Needs
 * aqt_workspace_bytes(AQT_OP_QUANTIZE_WEIGHTS, ., K, N, ., bits_w) of workspace.
 */
aqt_status aqt_quantize_weights(const float *w, int64_t K, int64_t N, int bits_w, void *wq_packed,
                                float *s_w, int8_t *wq_kn, uint32_t *clip_mask_w, void *ws,
                                size_t ws_bytes, void *stream, int32_t *dev_status);

/* Forward operand back to int8 codes [K,N] (a test aid; also the inverse the format promises). */
aqt_status aqt_unpack_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w,
                              int8_t *codes_kn, void *stream);

/*
 * The quantized dense layer on already-quantized operands (Sec. 1: integer
 * matmul; Sec. 2.2: de-quantize by multiplying with the scales):
 *   acc[m,n] = sum_k xq[m,k] * wq[k,n]                      (int32, exact)
 *   v[m,n]   = float(acc[m,n]) * (s_x * s_w[n]) (+ bias[n])
 *   y        = v | swish(v) | glu(v)
 * This is the serving form, and the unit the GEMM benchmark times.
 *   xq [M,K] int8; s_x device scalar; wq_packed as aqt_packed_weight_bytes();
 *   s_w [N]; bias nullable [N]; y [M,N] float32 ([M,N/2] for GLU);
 *   acc_out nullable [M,N] int32, the raw accumulators.
 * Requires K * qmax_x * qmax_w < 2^31, and < 2^31 / 16 for bits_w <= 4 (packed codes are
 * expanded to 16 * code on their way into the matrix cores); else AQT_ERR_UNSUPPORTED.
 * Needs aqt_workspace_bytes(AQT_OP_DENSE_FWD_Q, M, K, N, ., .) of workspace (K*N
 * bytes: the weight codes re-ordered for the matrix cores, rewritten per call).
 */
aqt_status aqt_dense_fwd_q(const int8_t *xq, const float *s_x, const void *wq_packed, const float *s_w,
                           int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                           int epilogue, float *y, int32_t *acc_out, void *ws, size_t ws_bytes,
                           void *stream);

/*
 * aqt_dense_fwd_q for callers that cannot allocate or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without acc_out and the workspace), same kernels, bit-identical y.
 * The scratch the contraction needs (the weight codes re-ordered for the matrix
 * cores, K * N bytes) lives in a static device array of AQT_STATIC_SCRATCH_BYTES
 * inside the library, one copy per GPU, held until the process ends; the call
 * allocates and frees nothing.  K * N above that size returns AQT_ERR_SCRATCH and
 * enqueues nothing.  The device the stream belongs to must be current.  All calls
 * on one GPU share the array (it keeps the last call's contents, every call
 * rewrites the part it reads): calls that overlap in time on one GPU, e.g. on two
 * streams, race; order them.
 */
#define AQT_STATIC_SCRATCH_BYTES (4u << 20) /* 4 MiB: up to K * N = 2048 * 2048 */
size_t aqt_static_scratch_bytes(void);
aqt_status aqt_dense_fwd_q_static(const int8_t *xq, const float *s_x, const void *wq_packed,
                                  const float *s_w, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w,
                                  const float *bias, int epilogue, float *y, void *stream);

/*
 * Producer-side abs-max for a chain of quantized layers.  The next layer's
 * activation quantizer (Fig. 2, per tensor) needs m = max|y| of this layer's
 * output before it can emit a single code; computing m where y is produced
 * saves that quantizer its first pass over y.
 * As aqt_dense_fwd_q (without acc_out), and additionally
 *   *y_absmax = max over all outputs of |y|   (device float, after bias / epilogue;
 *               for GLU over the [M,N/2] outputs).  Exactly the maximum of the
 *               values written to y; Inf or NaN in y gives Inf or NaN here.
 * The word is cleared by the call itself.
 */
aqt_status aqt_dense_fwd_q_absmax(const int8_t *xq, const float *s_x, const void *wq_packed,
                                  const float *s_w, int64_t M, int64_t K, int64_t N, int bits_x, int bits_w,
                                  const float *bias, int epilogue, float *y, float *y_absmax, void *ws,
                                  size_t ws_bytes, void *stream);

/*
 * Fig. 2 per tensor with m = max|x| supplied by the caller (device float, >= 0),
 * e.g. by aqt_dense_fwd_q_absmax: scale = m / qmax, codes as in aqt_quantize, one
 * pass over x.  Bit-identical to aqt_quantize(axis = AQT_AXIS_ALL) when m is the
 * true maximum; a smaller m saturates codes at +-qmax (clip_mask then has zeros),
 * a non-finite or negative m sets *dev_status to AQT_ERR_NONFINITE.
 */
aqt_status aqt_quantize_with_absmax(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                                    const float *absmax, int8_t *q, float *scale, uint32_t *clip_mask,
                                    void *stream, int32_t *dev_status);

/*
 * Weight-only modes (Sec. 4.1, configurations I8W and I4W: integer weights,
 * float32 activations; the weights are turned back into floats for the product):
 *   v[m,n] = (sum_k x[m,k] * wq[k,n]) * s_w[n] (+ bias[n]);  y = v | swish(v) | glu(v)
 *   x [M,K] float32; wq_packed, s_w as produced by aqt_quantize_weights; y float32
 *   [M,N] ([M,N/2] for GLU).
 * A float contraction: x is split into two bf16 terms (16 significant bits), the codes
 * are exact in bf16, accumulation is float32; every output lies within 1e-4 of the
 * sum of the magnitudes of its terms from the exact value (typically 1e-6).
 * Needs aqt_workspace_bytes(AQT_OP_DENSE_FWD_WONLY, ., K, N, ., .) of workspace.
 */
aqt_status aqt_dense_fwd_wonly(const float *x, const void *wq_packed, const float *s_w, int64_t M, int64_t K,
                               int64_t N, int bits_w, const float *bias, int epilogue, float *y, void *ws,
                               size_t ws_bytes, void *stream);

/*
 * The training forward: quantizes x per tensor and w per output channel inside
 * the call (weights are trained from scratch, so they are re-quantized every
 * step, Sec. 2.2), then runs aqt_dense_fwd_q.  Bit-identical to calling
 * aqt_quantize + aqt_quantize_weights + aqt_dense_fwd_q (Sec. 1: what is
 * trained is what is served).
 *   saved  nullable; when given, its non-null buffers receive xq, s_x, mask_x,
 *          wq_packed, wq_kn, s_w, mask_w for aqt_dense_bwd.  When NULL the codes
 *          live in the workspace only.
 */
aqt_status aqt_dense_fwd(const float *x, const float *w, int64_t M, int64_t K, int64_t N, int bits_x,
                         int bits_w, const float *bias, int epilogue, float *y, const aqt_saved *saved,
                         void *ws, size_t ws_bytes, void *stream, int32_t *dev_status);

/*
 * Straight-through backward of v = (s_x xq)(s_w wq) + bias with the scales held
 * constant (Fig. 2, stop_gradient):
 *   dx[m,k]  = mask_x[m,k] * sum_n (dy[m,n] * s_w[n]) * wq[k,n]
 *   dw[k,n]  = mask_w[k,n] * s_x * sum_m xq[m,k] * dy[m,n]
 *   dbias[n] = sum_m dy[m,n]
 * dy is the gradient with respect to v (epilogue AQT_EPI_NONE).  Any of dx, dw,
 * dbias may be NULL to skip it.  A NULL mask means "1 where the group's scale
 * is non-zero", which is what abs-max scaling always produces.  Results are
 * float32; the contractions run as two bf16 MFMA passes over a hi/lo split of
 * the float operand (codes are exact in bf16), accumulated in float32.
 * Uses saved->xq, s_x, wq_kn, s_w and the masks.
 */
aqt_status aqt_dense_bwd(const float *dy, const aqt_saved *saved, int64_t M, int64_t K, int64_t N,
                         int bits_x, int bits_w, float *dx, float *dw, float *dbias, void *ws,
                         size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AQT_H */
