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

__global__ void zero_f32_kernel(floatx4* p, long long n4) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) p[i] = zero4();
}

hipError_t launch_zero_f32(float* p, long long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const long long n4 = n / 4;
  hipLaunchKernelGGL(zero_f32_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<floatx4*>(p), n4);
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

__global__ void add_points_kernel(float* __restrict__ dst, const float* __restrict__ src, Idx d,
                                  Idx s, int nk, long long block4) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long long)nk * block4) return;
  long long pt = i / block4, e = i - pt * block4;
  const floatx4* sp = reinterpret_cast<const floatx4*>(src) + s.at(pt) * block4 + e;
  floatx4* dp = reinterpret_cast<floatx4*>(dst) + d.at(pt) * block4 + e;
  *dp = *dp + *sp;
}

hipError_t launch_add_points(float* dst, const float* src, Idx d, Idx s, int nk, long long block,
                             hipStream_t st) {
  if (nk <= 0) return hipSuccess;
  const long long block4 = block / 4;
  const long long n = (long long)nk * block4;
  prof_begin(7, st, nk);
  hipLaunchKernelGGL(add_points_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, dst,
                     src, d, s, nk, block4);
  prof_end(7, 0.0, 12.0 * (double)nk * (double)block, st);   // two reads and one write per float
  return hipGetLastError();
}

// Three-term bf16 form of an fp32 array (weights of the MGRIT_F32_BF16X3 path).
__global__ void split3_kernel(const float* __restrict__ src, unsigned short* __restrict__ dst,
                              long long n4) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const floatx4 v = reinterpret_cast<const floatx4*>(src)[i];
  ushort4 t[3];
  unsigned short* tp = reinterpret_cast<unsigned short*>(t);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const __bf16 h = (__bf16)v[e];
    const float r1 = v[e] - (float)h;
    const __bf16 m = (__bf16)r1;
    const __bf16 l = (__bf16)(r1 - (float)m);
    tp[e] = __builtin_bit_cast(unsigned short, h);
    tp[4 + e] = __builtin_bit_cast(unsigned short, m);
    tp[8 + e] = __builtin_bit_cast(unsigned short, l);
  }
#pragma unroll
  for (int k = 0; k < 3; ++k) reinterpret_cast<ushort4*>(dst + k * n4 * 4)[i] = t[k];
}

hipError_t launch_split3(const float* src, void* dst, long long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const long long n4 = n / 4;
  hipLaunchKernelGGL(split3_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, src,
                     (unsigned short*)dst, n4);
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
