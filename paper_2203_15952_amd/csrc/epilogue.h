// De-quantization epilogue pieces shared by the forward kernels.
#pragma once

#include <hip/hip_runtime.h>

namespace aqt {

// Logistic function.  One exp, of -|v| so that it cannot overflow, and one reciprocal
// of d = 1 + e, which lies in [1, 2]: the hardware estimate (1 ulp) plus one Newton
// step is within half an ulp there and needs none of the scaling an IEEE divide
// does.  Both signs take the same instructions, so mixed-sign wavefronts do not
// pay for two branches.  Total error stays under 4e-7 relative.
__device__ __forceinline__ float sigmoid_f32(float v) {
  const float e = expf(-fabsf(v));
  const float d = 1.0f + e;
  float r = __builtin_amdgcn_rcpf(d);
  r = fmaf(fmaf(-d, r, 1.0f), r, r);
  return (v >= 0.0f) ? r : e * r;
}

__device__ __forceinline__ float swish_f32(float v) { return v * sigmoid_f32(v); }

// Derivative factors for the backward through the activation, given sg = sigmoid of the
// argument the logistic function was applied to:
//   d swish(v) / dv = sg (1 + v (1 - sg));   d (a sigmoid(g)) / dg = a sg (1 - sg)
__device__ __forceinline__ float swish_dact_f32(float v, float sg) { return sg * (1.0f + v * (1.0f - sg)); }
__device__ __forceinline__ float glu_gate_dact_f32(float a, float sg) { return a * sg * (1.0f - sg); }

// Sec. 2.2: de-quantize by multiplying with the scales.  sc = s_x * s_w[n],
// rounded once; the int32 -> float32 conversion rounds to nearest even.
__device__ __forceinline__ float dequant_f32(int acc, float sc) { return static_cast<float>(acc) * sc; }

}  // namespace aqt
