// Few-row contraction for the dependent (serial) parts of the solve: the
// coarsest-level propagation and the serial scan advance only B rows per step,
// far too few for an MFMA tile, and every step waits for the previous one.  The
// work of one step is spread over as many workgroups as possible (a handful of
// output columns each) and computed with vector FMAs:
//   thread (row b, k-slice ks) accumulates  sum_k A[b][k] * Urow_u[k]  over its
//   interleaved float4 slices for the NU weight rows of the workgroup, partial
//   sums meet in LDS, and thread (b, column) applies the epilogue.
#pragma once
#include "gemm_core.h"

namespace mg {

constexpr int SK_NT = 256;       // threads per workgroup
constexpr int SK_MAXROWS = 32;   // rows per workgroup pass

// rows padded to a power of two <= 32
__host__ __device__ inline int sk_row_pad(int rows) {
  int p = 1;
  while (p < rows && p < SK_MAXROWS) p <<= 1;
  return p;
}

// Partial dot products of this thread.  getA(k) returns the float4 of the
// thread's row at columns k..k+3; urow[u] points at weight row u (K floats).
// rows_here <= Rp rows are live; idle threads return zeros.
template <int NU, class GetA>
__device__ inline void skinny_partial(float (&acc)[NU], int K, int ks, int ksl, bool live,
                                      const float* const (&urow)[NU], GetA getA) {
#pragma unroll
  for (int u = 0; u < NU; ++u) acc[u] = 0.f;
  if (!live) return;
  for (int k = ks * 4; k < K; k += ksl * 4) {
    const floatx4 a = getA(k);
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const floatx4 w = ldg4(urow[u] + k);
      acc[u] = fmaf(a[0], w[0], acc[u]);
      acc[u] = fmaf(a[1], w[1], acc[u]);
      acc[u] = fmaf(a[2], w[2], acc[u]);
      acc[u] = fmaf(a[3], w[3], acc[u]);
    }
  }
}

// red[(b*NU + u)*ksl + ks] holds the partials; returns the full sum for (b, u).
template <int NU>
__device__ inline float skinny_sum(const float* red, int b, int u, int ksl) {
  const float* p = red + (b * NU + u) * ksl;
  float s = 0.f;
  for (int i = 0; i < ksl; ++i) s += p[i];
  return s;
}

}  // namespace mg
