// De-quantization epilogue pieces shared by the forward kernels.
#pragma once

#include <hip/hip_runtime.h>

namespace aqt {

// Logistic function evaluated on the side where exp cannot overflow.
__device__ __forceinline__ float sigmoid_f32(float v) {
  if (v >= 0.0f) return 1.0f / (1.0f + expf(-v));
  const float e = expf(v);
  return e / (1.0f + e);
}

__device__ __forceinline__ float swish_f32(float v) { return v * sigmoid_f32(v); }

// Sec. 2.2: de-quantize by multiplying with the scales.  sc = s_x * s_w[n],
// rounded once; the int32 -> float32 conversion rounds to nearest even.
__device__ __forceinline__ float dequant_f32(int acc, float sc) { return static_cast<float>(acc) * sc; }

}  // namespace aqt
