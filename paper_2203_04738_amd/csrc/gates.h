// Gate nonlinearities shared by the step kernels.
#pragma once
#include <hip/hip_runtime.h>

namespace mg {

// Gate nonlinearities on the hardware exp2 / reciprocal units (each within 1 ulp):
// absolute error of sigmoid and tanh about 1e-7, far inside the fp32 parity bar,
// at a fraction of the instruction count of the library routines.
__device__ inline float fast_rcp(float a) { return __builtin_amdgcn_rcpf(a); }
__device__ inline float sigmoidf_(float a) {
  return fast_rcp(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * a));
}
__device__ inline float tanhf_(float a) {
  // tanh(a) = sign(a) (1 - e)/(1 + e), e = exp(-2|a|) in (0, 1]
  const float e = __builtin_amdgcn_exp2f(-2.88539008177792681f * fabsf(a));
  const float t = (1.0f - e) * fast_rcp(1.0f + e);
  return copysignf(t, a);
}

}  // namespace mg
