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
#define AQT_OP_DENSE_BWD_EPI 6         /* aqt_dense_bwd with an activation: M, K, N            */
#define AQT_OP_LAYERNORM_QUANTIZE 7    /* M rows; K = row length; N unused                     */
#define AQT_OP_FFN_FWD 8               /* M tokens, K = model width D, N = inner width H       */
#define AQT_OP_FFN_BWD 9
#define AQT_OP_DEPTHWISE_CONV_BWD 10   /* M = B * T tokens, K = channels C, N = kernel size kw  */
#define AQT_OP_CONV_MODULE_FWD 11      /* M = B * T tokens, K = model width D, N = kernel size  */
#define AQT_OP_CONV_MODULE_BWD 12
#define AQT_OP_MHSA_FWD 13             /* M = B * T tokens, K = model width D, N unused        */
#define AQT_OP_CONFORMER_LAYER_FWD 14  /* M = B * T tokens, K = model width D, N = inner width */
#define AQT_OP_ATTENTION_BWD 15        /* M = B * T tokens, K unused, N = heads                */
#define AQT_OP_LAYERNORM_BWD 16        /* M rows; K = row length; N unused                     */
#define AQT_OP_MHSA_BWD 17             /* M = B * T tokens, K = model width D, N = heads       */
#define AQT_OP_CONFORMER_LAYER_BWD 18  /* M = B * T tokens, K = model width D, N = inner width (heads <= 64, kernel <= 32 assumed) */

/* What the forward keeps for the backward.  All caller-owned device buffers. */
typedef struct aqt_saved {
  int8_t *xq;        /* [M,K] activation codes                                          */
  float *s_x;        /* [1]   activation scale                                          */
  uint32_t *mask_x;  /* nullable: ceil(M*K/32) words, bit i = element i, 1 = passes     */
  void *wq_packed;   /* forward operand, aqt_packed_weight_bytes(K,N,bits_w) bytes      */
  int8_t *wq_kn;     /* [K,N] weight codes in the layout of W (backward operand)        */
  float *s_w;        /* [N]   weight scales                                             */
  uint32_t *mask_w;  /* nullable: ceil(K*N/32) words over W's [K,N] order               */
  float *dact;       /* nullable: [M,N] derivative factors of the activation (Swish / GLU);  */
                     /* written by the forward when given, required by the backward then   */
  void *wprep;       /* nullable: the forward operand in matrix-core order (aqt_prepare_weights), */
                     /* read by the module calls of a layer whose policy says weights_ready    */
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
 * Serving with static weights: re-order the forward operand for the matrix cores once
 * (aqt_prepare_weights, into a caller buffer of aqt_prepared_weight_bytes()), then run
 * the contraction of Sec. 1 / Sec. 2.2 on it as often as needed with no workspace and no
 * per-call re-ordering pass.  Same arithmetic and bit-identical y as aqt_dense_fwd_q.
 * Needs a shape the matrix-core kernel takes: K a multiple of 128, N a multiple of 128
 * (N/2 a multiple of 64 for GLU), M >= 128; otherwise AQT_ERR_UNSUPPORTED (use
 * aqt_dense_fwd_q).  aqt_prepared_weight_bytes() is 0 for such shapes.  Packed (<= 4 bit)
 * weights stay two codes per byte in the prepared operand.
 */
size_t aqt_prepared_weight_bytes(int64_t K, int64_t N, int bits_w);
aqt_status aqt_prepare_weights(const void *wq_packed, int64_t K, int64_t N, int bits_w, void *wprep, void *stream);
aqt_status aqt_dense_fwd_q_prepared(const int8_t *xq, const float *s_x, const void *wprep, const float *s_w,
                                    int64_t M, int64_t K, int64_t N, int bits_x, int bits_w, const float *bias,
                                    int epilogue, float *y, void *stream);

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
 * Straight-through backward of out = act(v), v = (s_x xq)(s_w wq) + bias, with the scales
 * held constant (Fig. 2, stop_gradient):
 *   dv[m,n]  = dy[m, n mod out_cols] * dact[m,n]      (dv = dy when epilogue is AQT_EPI_NONE)
 *   dx[m,k]  = mask_x[m,k] * sum_n (dv[m,n] * s_w[n]) * wq[k,n]
 *   dw[k,n]  = mask_w[k,n] * s_x * sum_m xq[m,k] * dv[m,n]
 *   dbias[n] = sum_m dv[m,n]
 * dy is the gradient with respect to the layer's output: [M,N], or [M,N/2] for GLU.
 * With an activation (the Swish of the Conformer feed-forward module, the GLU of its
 * convolution module, Sec. 3.2) saved->dact must hold the factors the forward wrote:
 *   Swish: dact = s(v) (1 + v (1 - s(v)));   GLU: dact[m,j] = s(g), dact[m,j+N/2] = a s(g) (1 - s(g)),
 * s the logistic function, a / g the value / gate halves of v; the workspace is then
 * aqt_workspace_bytes(AQT_OP_DENSE_BWD_EPI, ...).  Any of dx, dw,
 * dbias may be NULL to skip it.  A NULL mask means "1 where the group's scale
 * is non-zero", which is what abs-max scaling always produces.  Results are
 * float32; the contractions run as two bf16 MFMA passes over a hi/lo split of
 * the float operand (codes are exact in bf16), accumulated in float32.
 * Uses saved->xq, s_x, wq_kn, s_w and the masks.
 */
aqt_status aqt_dense_bwd(const float *dy, const aqt_saved *saved, int64_t M, int64_t K, int64_t N,
                         int bits_x, int bits_w, int epilogue, float *dx, float *dw, float *dbias, void *ws,
                         size_t ws_bytes, void *stream);

/*
 * Layer normalisation of every row of x [M,D] (mean and biased variance over the row,
 * y = (x - mean) / sqrt(var + eps) * gamma + beta, float32; gamma / beta nullable) fused
 * with the per-tensor quantizer of Fig. 2 applied to y: the normalisation in front of the
 * Conformer feed-forward module (Sec. 3.2) feeds a quantized layer, so y itself is never
 * written.  Pass 1 takes the row statistics and max|y|; pass 2 re-forms y (same
 * arithmetic, same bits) and emits codes and scale exactly as aqt_quantize would on y.
 *   q [M,D] int8 and scale [1]: nullable together (then only y_out is produced);
 *   y_out nullable [M,D]: the normalised values themselves (for checking, or for a
 *   float consumer);  row_stats nullable [M,2]: mean and 1/sqrt(var + eps) per row.
 */
aqt_status aqt_layernorm_quantize(const float *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                                  float eps, int bits, int8_t *q, float *scale, float *y_out, float *row_stats,
                                  void *ws, size_t ws_bytes, void *stream, int32_t *dev_status);

/*
 * The product of the codes as "fake" quantization computes it on hardware without integer
 * matrix units (Sec. 1, Sec. 2.2): codes carried in float32, float32 multiply-accumulate
 * (the float32 matrix cores).  out[m,n] = sum_k float(xq[m,k]) * float(wq_kn[k,n]), exact
 * while every partial sum fits the 24-bit significand (K * qmax_x * qmax_w < 2^24), rounded
 * beyond.  A comparator for the native integer product of aqt_dense_fwd_q, not a path
 * of the layer.  xq [M,K], wq_kn [K,N] int8, out [M,N] float32.
 */
aqt_status aqt_fake_matmul_f32(const int8_t *xq, const int8_t *wq_kn, int64_t M, int64_t K, int64_t N,
                               float *out, void *stream);

/*
 * Per-layer precision (Sec. 4.1: configurations I8W, I4W, I8WA, I4WI8A, I4WA; Sec. 4.2 /
 * Table 2: int4 on chosen layers, int8 on the rest).  bits_x = 0 means float32
 * activations (the weight-only modes).
 */
typedef struct aqt_dense_policy {
  int bits_w;        /* 2..8 */
  int bits_x;        /* 2..8, or 0 = float32 activations */
  int weights_ready; /* 0: the call quantizes the float32 weights it is given (training: they change every step).
                        1: serving, what you train is what you serve: the layer's aqt_saved already holds
                        wq_packed and s_w (aqt_quantize_weights) and, if wprep is not NULL, the operand in
                        matrix-core order (aqt_prepare_weights); the float32 weight pointer is ignored and may
                        be NULL.  Module calls (aqt_ffn_fwd, aqt_mhsa_fwd, aqt_conv_module_fwd, the layer). */
} aqt_dense_policy;

/* The eight dense layers of one Conformer encoder layer (Sec. 3.2). */
typedef struct aqt_layer_policy {
  aqt_dense_policy ffn1_in, ffn1_out; /* first feed-forward module                           */
  aqt_dense_policy attn_qkv, attn_out; /* self-attention projections                          */
  aqt_dense_policy conv_pw1, conv_pw2; /* pointwise convolutions of the convolution module    */
  aqt_dense_policy ffn2_in, ffn2_out; /* second feed-forward module                          */
} aqt_layer_policy;

#define AQT_POLICY_ALL 0              /* every layer at bits_w (Table 2: E1 int8, E3 int4)       */
#define AQT_POLICY_EXCEPT_FIRST_LAST 1 /* first and last encoder layer stay int8 (E6)              */
#define AQT_POLICY_EXCEPT_ATTENTION 2  /* self-attention projections stay int8 (E7)                */
#define AQT_POLICY_FIRST_K 3           /* only the first k encoder layers get bits_w (E8 - E13)    */

/*
 * Fill out[0..n_layers) (host memory) with one of Table 2's patterns: layers the pattern
 * selects get bits_w weights, all others int8 weights; every layer gets bits_x activations.
 * k is only used by AQT_POLICY_FIRST_K.
 */
aqt_status aqt_policy_preset(int pattern, int n_layers, int k, int bits_w, int bits_x, aqt_layer_policy *out);

/*
 * Bytes the quantized weights of n_layers encoder layers take under a policy (packed codes
 * plus one float32 scale per output channel; model width d_model, feed-forward width d_ff):
 * the model-size side of Table 2's trade-off.  Host computation.
 */
size_t aqt_policy_weight_bytes(const aqt_layer_policy *policy, int n_layers, int64_t d_model, int64_t d_ff);

/* What the feed-forward module keeps for its backward.  Caller-owned device buffers. */
typedef struct aqt_ffn_saved {
  aqt_saved l1;     /* first layer  [M,D] x [D,H]; l1.dact [M,H] required for aqt_ffn_bwd         */
  aqt_saved l2;     /* second layer [M,H] x [H,D]                                                 */
  float *h;         /* [M,H] output of the first layer after Swish                                */
  float *xn;        /* [M,D] normalised input in float32: required when policy[0].bits_x == 0     */
  float *row_stats; /* nullable [M,2]: mean and reciprocal standard deviation of every input row */
} aqt_ffn_saved;

/*
 * The Conformer feed-forward module (Sec. 3.2) on quantized layers, as one call:
 *   xn = layernorm(x);  h = swish(dense(xn, w1) + b1);  y = dense(h, w2) + b2
 * with each dense layer at its policy[i] precision (policy[0]: first layer, policy[1]:
 * second).  Integer activations: the normalisation is fused with the first quantizer
 * (aqt_layernorm_quantize), the first contraction emits max|h| and the second quantizer
 * runs in one pass (aqt_dense_fwd_q_absmax, aqt_quantize_with_absmax).  Float32
 * activations (bits_x = 0) take aqt_dense_fwd_wonly.
 *   x [M,D]; w1 [D,H], b1 nullable [H]; w2 [H,D], b2 nullable [D]; y [M,D].
 */
aqt_status aqt_ffn_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps,
                       const float *w1, const float *b1, const float *w2, const float *b2, int64_t M, int64_t D,
                       int64_t H, const aqt_dense_policy *policy, float *y, const aqt_ffn_saved *saved, void *ws,
                       size_t ws_bytes, void *stream, int32_t *dev_status);

/*
 * Straight-through backward of aqt_ffn_fwd down to the normalised input:
 *   dxn [M,D] (gradient with respect to layernorm(x)), dw1 [D,H], db1 [H], dw2 [H,D], db2 [D];
 * any of them may be NULL.  Needs integer activations in both layers (a weight-only layer's
 * weight gradient contracts two float tensors, which this library does not do) and the
 * buffers aqt_ffn_fwd filled.  The normalisation's own backward is left to the caller.
 */
aqt_status aqt_ffn_bwd(const float *dy, const aqt_ffn_saved *saved, int64_t M, int64_t D, int64_t H,
                       const aqt_dense_policy *policy, float *dxn, float *dw1, float *db1, float *dw2,
                       float *db2, void *ws, size_t ws_bytes, void *stream);

/*
 * Depthwise convolution along time, the float layer between the two pointwise convolutions
 * of the Conformer convolution module (Sec. 3.2: kernel size 32; Sec. 3.3: causal, kernel
 * size 15; convolution kernels stay unquantized), with what follows it fused in:
 *   v[b,t,c]   = bias[c] + sum_j w[j,c] * x[b, t + j - pad_left, c]     (frames outside [0,T) are zero)
 *   n          = v * norm_scale[c] + norm_shift[c]        (the normalisation with fixed statistics)
 *   out        = swish ? n * sigmoid(n) : n
 * x, out [B,T,C] (B utterances of T frames, C contiguous); w [kw,C]; bias, norm_scale,
 * norm_shift nullable [C]; 0 <= pad_left < kw (kw - 1: causal).  dfac nullable [B,T,C]:
 * d out / d v, what the backward needs.  out_absmax nullable device float: max|out|, cleared
 * by the call, for aqt_quantize_with_absmax in front of the next quantized layer.
 */
aqt_status aqt_depthwise_conv_fwd(const float *x, int64_t B, int64_t T, int64_t C, const float *w, const float *bias,
                                  int kw, int pad_left, const float *norm_scale, const float *norm_shift, int swish,
                                  float *out, float *dfac, float *out_absmax, void *stream);

/*
 * Gradients of aqt_depthwise_conv_fwd for the upstream gradient dout [B,T,C]; with
 * dv = dout * dfac (dfac nullable: dv = dout):
 *   dx[b,u,c] = sum_j w[j,c] * dv[b, u - j + pad_left, c];   dw[j,c] = sum_{b,t} dv[b,t,c] * x[b, t + j - pad_left, c];
 *   dbias[c]  = sum_{b,t} dv[b,t,c].
 * Any of dx, dw, dbias may be NULL (x is only read for dw).  The sums over tokens are folded
 * in a fixed order.  Workspace: aqt_workspace_bytes(AQT_OP_DEPTHWISE_CONV_BWD, B*T, C, kw, ., .)
 * for dw / dbias.  Gradients of norm_scale / norm_shift are not produced.
 */
aqt_status aqt_depthwise_conv_bwd(const float *dout, const float *dfac, const float *x, const float *w, int64_t B,
                                  int64_t T, int64_t C, int kw, int pad_left, float *dx, float *dw, float *dbias,
                                  void *ws, size_t ws_bytes, void *stream);

/* What the convolution module keeps for its backward.  Caller-owned device buffers. */
typedef struct aqt_conv_saved {
  aqt_saved pw1;    /* first pointwise convolution [M,D] x [D,2D] with GLU; pw1.dact [M,2D] for the backward */
  aqt_saved pw2;    /* second pointwise convolution [M,D] x [D,D]                                            */
  float *g;         /* [M,D] output of the GLU = input of the depthwise convolution                          */
  float *s;         /* [M,D] after depthwise convolution, normalisation and Swish                            */
  float *dfac;      /* nullable [M,D]: d s / d (depthwise result), needed by aqt_conv_module_bwd            */
  float *row_stats; /* nullable [M,2]: mean and reciprocal standard deviation of every input row             */
} aqt_conv_saved;

/*
 * The Conformer convolution module (Sec. 3.2) as one call, M = B * T tokens of width D:
 *   xn = layernorm(x);  g = glu(dense(xn, w1) + b1);  s = swish(norm(depthwise(g)));  y = dense(s, w2) + b2
 * The pointwise convolutions are quantized dense layers at policy[0] / policy[1] (integer
 * activations only); the depthwise convolution and the normalisation behind it stay float32
 * (Sec. 3.3).  Fused as in aqt_ffn_fwd: normalisation with the first quantizer, and the
 * depthwise kernel emits max|s| so the second quantizer runs in one pass.
 *   w1 [D,2D] (value columns first, gate columns second), b1 nullable [2D]; w_dw [kw,D], b_dw,
 *   norm_scale, norm_shift nullable [D]; w2 [D,D], b2 nullable [D]; y [M,D].
 */
aqt_status aqt_conv_module_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps,
                               const float *w1, const float *b1, const float *w_dw, const float *b_dw,
                               const float *norm_scale, const float *norm_shift, const float *w2, const float *b2,
                               int64_t B, int64_t T, int64_t D, int kw, int pad_left, const aqt_dense_policy *policy,
                               float *y, const aqt_conv_saved *saved, void *ws, size_t ws_bytes, void *stream,
                               int32_t *dev_status);

/*
 * Straight-through backward of aqt_conv_module_fwd down to the normalised input:
 *   dxn [M,D], dw1 [D,2D], db1 [2D], dw_dw [kw,D], db_dw [D], dw2 [D,D], db2 [D]; any may be NULL.
 * The normalisation's own backward is left to the caller.
 */
aqt_status aqt_conv_module_bwd(const float *dy, const aqt_conv_saved *saved, const float *w_dw, int64_t B, int64_t T,
                               int64_t D, int kw, int pad_left, const aqt_dense_policy *policy, float *dxn,
                               float *dw1, float *db1, float *dw_dw, float *db_dw, float *dw2, float *db2, void *ws,
                               size_t ws_bytes, void *stream);

/*
 * The float core of the self-attention module (Sec. 3.2: 4 or 8 heads; Sec. 3.3: limited
 * left and right context): for every utterance b, head h and query frame t, over the key
 * frames j of the same utterance with t - left_context <= j <= t + right_context (a negative
 * limit: none on that side),
 *   p = softmax_j( q_t . k_j / sqrt(dh) ),   ctx[b,t,h*dh + d] = sum_j p_j v_j[d],   dh = D / heads.
 * qkv [B*T, 3D]: queries, keys, values in three column blocks of width D (the output of the
 * fused projection), head h in columns h*dh .. (h+1)*dh of each block; ctx [B*T, D].
 * dh <= 64.  Float32 with an online softmax; the scores are not written anywhere.
 * ctx_absmax nullable device float: max|ctx|, cleared by the call, for
 * aqt_quantize_with_absmax in front of the output projection.
 * lse nullable [B*T, heads]: log2 of the softmax's normaliser, in the units the kernel keeps
 * its scores in (so that p_j = 2^(score_j - lse)); what aqt_attention_bwd needs.
 */
aqt_status aqt_attention_fwd(const float *qkv, int64_t B, int64_t T, int64_t D, int heads, int left_context,
                             int right_context, float *ctx, float *ctx_absmax, float *lse, void *stream);

/*
 * Gradient of aqt_attention_fwd with respect to qkv for the upstream gradient dctx [B*T, D]:
 * the chain rule through the softmax and the two products, on the float32 matrix cores, the
 * probabilities formed again from qkv and lse.  qkv, ctx and lse as the forward left them;
 * dqkv [B*T, 3D] in the layout of qkv, every element written.  Each sum has one fixed order
 * (no atomics).  Workspace: aqt_workspace_bytes(AQT_OP_ATTENTION_BWD, B*T, ., heads, ., .).
 */
aqt_status aqt_attention_bwd(const float *qkv, const float *ctx, const float *dctx, const float *lse, int64_t B,
                             int64_t T, int64_t D, int heads, int left_context, int right_context, float *dqkv,
                             void *ws, size_t ws_bytes, void *stream);

/* Buffers of the self-attention module.  Caller-owned device memory. */
typedef struct aqt_mhsa_saved {
  aqt_saved qkv;    /* fused query / key / value projection [M,D] x [D,3D] */
  aqt_saved out;    /* output projection [M,D] x [D,D]                     */
  float *qkv_f;     /* [M,3D] projected queries, keys, values              */
  float *ctx;       /* [M,D] attention result                              */
  float *row_stats; /* nullable [M,2]                                      */
  float *lse;       /* nullable [M,heads]: the softmax normalisers, for the backward */
} aqt_mhsa_saved;

/*
 * The self-attention module (Sec. 3.2) as one call, forward, M = B * T tokens of width D:
 *   xn = layernorm(x);  qkv = dense(xn, wqkv) + bqkv;  ctx = attention(qkv);  y = dense(ctx, wo) + bo
 * with the projections as quantized dense layers at policy[0] / policy[1] (integer
 * activations; Table 2's E7 keeps exactly these two layers at int8) and the attention itself in
 * float32 (the paper quantizes the layers' weights and inputs, not the score products).
 * Fused like the other modules: normalisation with the first quantizer, max|ctx| from the
 * attention kernel for a one-pass second quantizer.  With saved->lse given, the softmax
 * normalisers are kept for aqt_mhsa_bwd.
 */
aqt_status aqt_mhsa_fwd(const float *x, const float *ln_gamma, const float *ln_beta, float ln_eps, const float *wqkv,
                        const float *bqkv, const float *wo, const float *bo, int64_t B, int64_t T, int64_t D,
                        int heads, int left_context, int right_context, const aqt_dense_policy *policy, float *y,
                        const aqt_mhsa_saved *saved, void *ws, size_t ws_bytes, void *stream, int32_t *dev_status);

/* out[i] = x[i] + alpha * m[i], i < n: the residual connection around a module (float32,
 * two roundings per element; out may alias x or m). */
aqt_status aqt_residual_add(const float *x, const float *m, float alpha, float *out, int64_t n, void *stream);

/* Weights of one Conformer encoder layer (Sec. 3.2), device pointers, float32; layouts as in
 * aqt_ffn_fwd, aqt_mhsa_fwd and aqt_conv_module_fwd.  Every *_ln_*, bias and norm pointer
 * may be NULL. */
typedef struct aqt_conformer_layer_weights {
  const float *ffn1_ln_g, *ffn1_ln_b, *ffn1_w1, *ffn1_b1, *ffn1_w2, *ffn1_b2;
  const float *att_ln_g, *att_ln_b, *att_wqkv, *att_bqkv, *att_wo, *att_bo;
  const float *conv_ln_g, *conv_ln_b, *conv_w1, *conv_b1, *conv_wdw, *conv_bdw, *conv_norm_scale,
      *conv_norm_shift, *conv_w2, *conv_b2;
  const float *ffn2_ln_g, *ffn2_ln_b, *ffn2_w1, *ffn2_b1, *ffn2_w2, *ffn2_b2;
  const float *out_ln_g, *out_ln_b;
} aqt_conformer_layer_weights;

typedef struct aqt_conformer_layer_shape {
  int64_t B, T, D, H;                 /* utterances, frames, model width, feed-forward width     */
  int heads, kw, pad_left;            /* attention heads; depthwise kernel size and left padding  */
  int left_context, right_context;    /* attention window, negative: unlimited                    */
  float ln_eps;
} aqt_conformer_layer_shape;

/* Buffers of one encoder layer.  Caller-owned device memory. */
typedef struct aqt_conformer_layer_saved {
  aqt_ffn_saved ffn1, ffn2;
  aqt_mhsa_saved att;
  aqt_conv_saved conv;
  float *r1, *r2, *r3, *r4;   /* [M,D] each: the residual stream after each module */
  float *m;                   /* [M,D] module output before it joins the stream     */
  float *out_row_stats;       /* nullable [M,2]: statistics of the final normalisation, for the backward */
} aqt_conformer_layer_saved;

/*
 * One Conformer encoder layer (Sec. 3.2), forward, with every dense layer at the precision
 * its aqt_layer_policy entry names (Sec. 4.2 / Table 2):
 *   r1 = x + ffn(x) / 2;  r2 = r1 + mhsa(r1);  r3 = r2 + conv(r2);  r4 = r3 + ffn(r3) / 2;  y = layernorm(r4)
 * x, y [B*T, D].  The self-attention and convolution modules need integer activations.  For
 * aqt_conformer_layer_bwd the saved buffers must include every row_stats, out_row_stats, att.lse,
 * conv.dfac and the dact buffers of the layers with an activation.  Errors: every module's argument,
 * policy, buffer and workspace check runs before the first launch, so a refused call has written nothing.
 */
aqt_status aqt_conformer_layer_fwd(const float *x, const aqt_conformer_layer_weights *w,
                                   const aqt_conformer_layer_shape *shape, const aqt_layer_policy *policy, float *y,
                                   const aqt_conformer_layer_saved *saved, void *ws, size_t ws_bytes, void *stream,
                                   int32_t *dev_status);

/*
 * Backward of the layer normalisation of aqt_layernorm_quantize (the quantizer behind it passes
 * gradients straight through): with xh = (x - mean) rstd and g = dy gamma,
 *   dx = add + (g - mean_row(g) - xh mean_row(g xh)) rstd;   dgamma = sum_m dy xh;   dbeta = sum_m dy.
 * x, dy, dx [M,D]; row_stats [M,2] as the forward stored them; gamma nullable (ones); add nullable
 * [M,D]: a gradient to add in (the one arriving over a residual connection); dgamma / dbeta
 * nullable [D], summed in a fixed order.  Workspace: aqt_workspace_bytes(AQT_OP_LAYERNORM_BWD, M, D, ., ., .).
 */
aqt_status aqt_layernorm_bwd(const float *x, const float *row_stats, const float *gamma, const float *dy,
                             const float *add, int64_t M, int64_t D, float *dx, float *dgamma, float *dbeta,
                             void *ws, size_t ws_bytes, void *stream);

/*
 * Straight-through backward of aqt_mhsa_fwd down to the normalised input:
 *   dxn [M,D], dwqkv [D,3D], dbqkv [3D], dwo [D,D], dbo [D]; any may be NULL.
 * Needs saved->lse and the buffers aqt_mhsa_fwd filled.
 */
aqt_status aqt_mhsa_bwd(const float *dy, const aqt_mhsa_saved *saved, int64_t B, int64_t T, int64_t D, int heads,
                        int left_context, int right_context, const aqt_dense_policy *policy, float *dxn,
                        float *dwqkv, float *dbqkv, float *dwo, float *dbo, void *ws, size_t ws_bytes, void *stream);

/* Gradients of one encoder layer's weights: the fields of aqt_conformer_layer_weights, writable; NULL = not wanted. */
typedef struct aqt_conformer_layer_grads {
  float *ffn1_ln_g, *ffn1_ln_b, *ffn1_w1, *ffn1_b1, *ffn1_w2, *ffn1_b2;
  float *att_ln_g, *att_ln_b, *att_wqkv, *att_bqkv, *att_wo, *att_bo;
  float *conv_ln_g, *conv_ln_b, *conv_w1, *conv_b1, *conv_wdw, *conv_bdw, *conv_norm_scale, *conv_norm_shift,
      *conv_w2, *conv_b2;
  float *ffn2_ln_g, *ffn2_ln_b, *ffn2_w1, *ffn2_b1, *ffn2_w2, *ffn2_b2;
  float *out_ln_g, *out_ln_b;
} aqt_conformer_layer_grads;

/*
 * Straight-through backward of aqt_conformer_layer_fwd (training form: weights_ready = 0, integer
 * activations everywhere): dx [M,D] and the weight gradients asked for.  x and w as in the forward
 * call, saved as it left them (including every row_stats, out_row_stats, att.lse, conv.dfac and the
 * dact buffers).  conv_norm_scale / conv_norm_shift gradients are not produced (fixed statistics)
 * and must be NULL.  As in the forward, every check runs before the first launch.
 */
aqt_status aqt_conformer_layer_bwd(const float *dy, const float *x, const aqt_conformer_layer_weights *w,
                                   const aqt_conformer_layer_shape *shape, const aqt_layer_policy *policy,
                                   const aqt_conformer_layer_saved *saved, float *dx,
                                   const aqt_conformer_layer_grads *grads, void *ws, size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AQT_H */
