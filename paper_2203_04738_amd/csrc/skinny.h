// Few-row contraction for the dependent (serial) parts of the solve: the
// coarsest-level propagation and the serial scan advance only B rows per step,
// far too few for an MFMA tile, and every step waits for the previous one.  The
// work of one step is spread over as many workgroups as possible (a handful of
// output columns each) and computed with vector FMAs:
//   thread (row b, k-slice ks) accumulates  sum_k A[b][k] * Urow_u[k]  over its
//   interleaved float4 slices for the NU weight rows of the workgroup, partial
//   sums meet in LDS, and thread (b, column) applies the epilogue.
#pragma once
#include "gemm_core_bf16.h"

namespace mg {

constexpr int SK_NT = 1024;      // threads per workgroup
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
template <int NU, class WT, class GetA>
__device__ inline void skinny_partial(float (&acc)[NU], int K, int ks, int ksl, bool live,
                                      const WT* const (&urow)[NU], GetA getA) {
  // several independent slices are fetched before any is consumed, so that the
  // loop pays one memory round trip per UNR slices
  constexpr int UNR = NU >= 12 ? 1 : (NU >= 5 ? 2 : 4);
#pragma unroll
  for (int u = 0; u < NU; ++u) acc[u] = 0.f;
  if (!live) return;
  const int stride = ksl * 4;
  for (int k = ks * 4; k < K; k += stride * UNR) {
    floatx4 a[UNR];
    floatx4 w[UNR][NU];
#pragma unroll
    for (int i = 0; i < UNR; ++i) {
      const int kk = k + i * stride;
      if (kk < K) {
        a[i] = getA(kk);
#pragma unroll
        for (int u = 0; u < NU; ++u) w[i][u] = ldg4w(urow[u] + kk);
      } else {
        a[i] = zero4();
#pragma unroll
        for (int u = 0; u < NU; ++u) w[i][u] = zero4();
      }
    }
#pragma unroll
    for (int i = 0; i < UNR; ++i)
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        acc[u] = fmaf(a[i][0], w[i][u][0], acc[u]);
        acc[u] = fmaf(a[i][1], w[i][u][1], acc[u]);
        acc[u] = fmaf(a[i][2], w[i][u][2], acc[u]);
        acc[u] = fmaf(a[i][3], w[i][u][3], acc[u]);
      }
  }
}

// Combine the partials of all k-slices of a row.  ks is the fast thread index, so
// the slices of one row occupy min(ksl, 64) consecutive lanes of a wave: those are
// summed with lane shuffles, and one lane per segment leaves the segment sum in
// red[(b*NU + u)*nseg + seg], nseg = ksl / min(ksl, 64) <= SK_NT/64.
__device__ inline int sk_nseg(int ksl) { return ksl > 64 ? ksl / 64 : 1; }

template <int NU>
__device__ inline void skinny_reduce(float (&acc)[NU], float* red, int bl, int ks, int ksl) {
  const int width = ksl > 64 ? 64 : ksl;
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    float v = acc[u];
    for (int off = width >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    acc[u] = v;
  }
  if ((ks & (width - 1)) == 0) {
    const int nseg = sk_nseg(ksl);
#pragma unroll
    for (int u = 0; u < NU; ++u) red[(bl * NU + u) * nseg + ks / width] = acc[u];
  }
}

template <int NU>
__device__ inline float skinny_sum(const float* red, int b, int u, int ksl) {
  const int nseg = sk_nseg(ksl);
  const float* p = red + (b * NU + u) * nseg;
  float s = 0.f;
  for (int i = 0; i < nseg; ++i) s += p[i];
  return s;
}

}  // namespace mg
