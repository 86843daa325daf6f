// Few-row contraction for the dependent (serial) parts of the solve: the
// coarsest-level propagation and the serial scan advance only B rows per step,
// far too few for an MFMA tile, and every step waits for the previous one, so
// what counts is the latency of one step.  The work of a step is spread over
// some hundreds of workgroups (a block of rows x a handful of output columns
// each) and computed with vector FMAs:
//   thread (row group rg, k-slice ks) accumulates  sum_k A[row][k] * W_u[k]  for
//   its RR rows and the NU weight rows of the workgroup over its float4 slices
//   (weights are loaded once per RR rows), the RR*NU partial sums of all k-slices
//   are combined by a halving butterfly over lanes plus a short LDS pass, and
//   thread (row, column) applies the epilogue.
// Weights may be float or bf16 (WT); the arithmetic is fp32 either way.
#pragma once
#include "gemm_core_bf16.h"

namespace mg {

constexpr int SK_RR = 4;          // rows register-blocked per thread
constexpr int SK_MAXNT = 1024;    // largest workgroup
constexpr int SK_MAXROWS = 32;    // largest row block of a workgroup

constexpr int sk_pow2_ceil(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}

// Launch geometry shared by host and device: rows of a workgroup are split into
// Gp (power of two) groups of SK_RR rows; each group has ksl (power of two)
// k-slices; the workgroup has Gp * ksl threads (at least 64).
struct SkGeom {
  int Gp, ksl, nt;
};
__host__ __device__ inline SkGeom sk_geom(int rows_block, int K) {
  SkGeom g;
  const int ngrp = (rows_block + SK_RR - 1) / SK_RR;
  g.Gp = 1;
  while (g.Gp < ngrp) g.Gp <<= 1;
  const int chunks = K / 4;
  int ksl = 1;
  while (ksl * 2 <= chunks && ksl * 2 * g.Gp <= SK_MAXNT) ksl <<= 1;
  while (ksl * g.Gp < 64) ksl <<= 1;
  g.ksl = ksl;
  g.nt = ksl * g.Gp;
  return g;
}

// Partial dot products of this thread: acc[i][u] = sum over its k-slices of
// A_i[k] * W_u[k].  getA(i, k) returns the float4 of the thread's i-th row at
// columns k..k+3; wrow[u] points at weight row u (K elements).
template <int NU, class WT, class GetA>
__device__ inline void skinny_dot(float (&acc)[SK_RR][NU], int K, int ks, int ksl,
                                  const WT* const (&wrow)[NU], GetA getA) {
#pragma unroll
  for (int i = 0; i < SK_RR; ++i)
#pragma unroll
    for (int u = 0; u < NU; ++u) acc[i][u] = 0.f;
  for (int k = ks * 4; k < K; k += ksl * 4) {
    floatx4 a[SK_RR];
    floatx4 w[NU];
#pragma unroll
    for (int i = 0; i < SK_RR; ++i) a[i] = getA(i, k);
#pragma unroll
    for (int u = 0; u < NU; ++u) w[u] = ldg4w(wrow[u] + k);
#pragma unroll
    for (int i = 0; i < SK_RR; ++i)
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        acc[i][u] = fmaf(a[i][0], w[u][0], acc[i][u]);
        acc[i][u] = fmaf(a[i][1], w[u][1], acc[i][u]);
        acc[i][u] = fmaf(a[i][2], w[u][2], acc[i][u]);
        acc[i][u] = fmaf(a[i][3], w[u][3], acc[i][u]);
      }
  }
}

// Sum VP values (a power of two >= SK_RR*NU) over the k-slices of a row group.  ks is
// the fast thread index, so the slices of one group occupy W = min(ksl, 64)
// consecutive lanes of a wave.  Halving butterfly: at step s (lane distance 2^s) a
// lane hands half of its remaining values to its partner and adds the half it
// receives, so the sums end up spread over the lanes with VP - 1 exchanges instead of
// VP * log2(W); once a lane is down to one value the remaining steps are plain
// exchanges.  The lane that ends up with value idx leaves it in
// red[(rg * nseg + seg) * VP + idx], seg = ks / W.
template <int VP, int S>
__device__ inline void skinny_reduce_step(float (&v)[VP], int lane, int W, int& idx, int& nv) {
  constexpr int off = 1 << S;
  constexpr int cur = (VP >> S) > 0 ? (VP >> S) : 1;     // values owned before this step
  if (off >= W) return;
  if constexpr (cur > 1) {
    constexpr int half = cur / 2;
    const bool up = (lane & off) != 0;
#pragma unroll
    for (int i = 0; i < half; ++i) {
      const float send = up ? v[i] : v[half + i];
      const float keep = up ? v[half + i] : v[i];
      v[i] = keep + __shfl_xor(send, off, 64);
    }
    idx = idx * 2 + (up ? 1 : 0);
    nv = half;
  } else {
    v[0] += __shfl_xor(v[0], off, 64);
  }
}

template <int VP>
__device__ inline void skinny_reduce(float (&v)[VP], float* red, int rg, int ks, int ksl) {
  const int W = ksl > 64 ? 64 : ksl;
  const int lane = threadIdx.x & 63;
  int idx = 0;       // index of this lane's block of values, in units of its block size
  int nv = VP;       // values this lane still owns
  skinny_reduce_step<VP, 0>(v, lane, W, idx, nv);
  skinny_reduce_step<VP, 1>(v, lane, W, idx, nv);
  skinny_reduce_step<VP, 2>(v, lane, W, idx, nv);
  skinny_reduce_step<VP, 3>(v, lane, W, idx, nv);
  skinny_reduce_step<VP, 4>(v, lane, W, idx, nv);
  skinny_reduce_step<VP, 5>(v, lane, W, idx, nv);
  // lanes beyond the first VP of a group hold replicas (only when VP < W)
  const int lw = lane & (W - 1);
  if (lw < VP) {
    const int nseg = ksl > 64 ? ksl / 64 : 1;
    float* dst = red + (rg * nseg + ks / W) * VP + idx * nv;
#pragma unroll
    for (int i = 0; i < VP; ++i)
      if (i < nv) dst[i] = v[i];
  }
}

template <int VP>
__device__ inline float skinny_sum(const float* red, int rg, int idx, int ksl) {
  const int nseg = ksl > 64 ? ksl / 64 : 1;
  const float* p = red + (rg * nseg) * VP + idx;
  float s = 0.f;
  for (int i = 0; i < nseg; ++i) s += p[i * VP];
  return s;
}

}  // namespace mg
