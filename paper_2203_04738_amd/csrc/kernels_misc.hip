// Small streaming kernels: accumulator clearing, coarse-point copies (the
// injection / correction transfers of Alg. 2 line 5 at coarse points) and the
// final square root of the residual accumulators.
#include "common.h"
#include "gemm_core.h"

namespace mg {

__global__ void fill_f64_kernel(double* p, long long n, double v) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_fill_f64(double* p, long long n, double v, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_f64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

// One float4 per thread; `block` (floats per point) is a multiple of 4.
__global__ void copy_points_kernel(float* __restrict__ dst, const float* __restrict__ src, Idx d,
                                   Idx s, int nk, long long block4) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)nk * block4) return;
  long long pt = i / block4, e = i - pt * block4;
  const floatx4* sp = reinterpret_cast<const floatx4*>(src) + s.at(pt) * block4 + e;
  floatx4* dp = reinterpret_cast<floatx4*>(dst) + d.at(pt) * block4 + e;
  *dp = *sp;
}

hipError_t launch_copy_points(float* dst, const float* src, Idx d, Idx s, int nk, long long block,
                              hipStream_t st) {
  if (nk <= 0) return hipSuccess;
  const long long block4 = block / 4;
  const long long n = (long long)nk * block4;
  prof_begin(7, st, nk);
  hipLaunchKernelGGL(copy_points_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dst,
                     src, d, s, nk, block4);
  prof_end(7, 0.0, 8.0 * (double)nk * (double)block, st);   // one read and one write per float
  return hipGetLastError();
}

__global__ void sqrt_to_float_kernel(const double* acc, float* out, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (float)sqrt(acc[i]);
}

hipError_t launch_sqrt_to_float(const double* acc, float* out, int n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(sqrt_to_float_kernel, dim3((n + 255) / 256), dim3(256), 0, s, acc, out, n);
  return hipGetLastError();
}

}  // namespace mg
