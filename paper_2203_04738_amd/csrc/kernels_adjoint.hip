// Adjoint kernels: the fused transposed-Jacobian level step
//   w_out = k_d*w + U_r^T(k_r*w) + U_z^T(k_z*w) + U_n^T(k_q*w)
// (discrete adjoint of Eq. 16 / Eq. 3, Appendix A.2) with the same MGRIT
// epilogues as the forward step, the transposition of U it contracts with, and
// the parameter-gradient reductions of Alg. 3's gradient line.
#include "common.h"
#include "gemm_core.h"
#include "gemm_core_bf16.h"
#include "skinny.h"

namespace mg {

// ---------------------------------------------------------------------------
// Adjoint level step: out[R,H] = (kap[:, 0:3H] * (w,w,w))[R,3H] . UT[H,3H]^T + k_d*w
// ---------------------------------------------------------------------------
// Operands of one output element that do not depend on the contraction.
struct AdjEpiIn {
  float kd, wv, gval, cur;
};
// Element offsets (column 0) of one row of a launch: input adjoint, coefficient row,
// out/cur/g, coarse array.  Computed once per tile row and kept in LDS.
struct AdjRow {
  long long in, k, o, a;
};
__device__ inline AdjRow adj_row(const AdjArgs& a, long long r) {
  const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
  const int b = (int)(r - pt * a.B);
  AdjRow ro;
  ro.in = (a.in.at(pt) * a.B + b) * a.H;
  ro.k = (a.k.at(pt) * a.B + b) * (long long)a.kw;
  ro.o = (a.o.at(pt) * a.B + b) * a.H;
  ro.a = (a.a.at(pt) * a.B + b) * a.H;
  // (row offsets are multiples of four elements: bit 0 marks the coarse points of ff_cf / ff_rem)
  if (a.ff_cf > 0 && a.a.at(pt) % a.ff_cf == a.ff_rem) ro.a |= 1;
  return ro;
}

template <int MODE>
__device__ inline AdjEpiIn adj_epi_load(const AdjArgs& a, const AdjRow& ro, int j) {
  AdjEpiIn e;
  e.kd = a.kap[ro.k + 3 * a.H + j];
  e.wv = a.w_in[ro.in + j];
  const long long oi = ro.o + j;
  e.gval = a.g ? a.g[oi] : 0.f;
  e.cur = MODE == STEP_RESID ? a.w[oi] : 0.f;
  return e;
}

// Output of one element of the adjoint step: row (point pt, batch b), column j, given
// the contraction  sum_g (U_g^T (k_g * w))_j.
template <int MODE>
__device__ inline void adj_epi_finish(const AdjArgs& a, const AdjRow& ro, int j, float dot,
                                      const AdjEpiIn& e, double& nrm) {
  const float wn = e.kd * e.wv + dot;
  const long long oi = ro.o + j;
  if (MODE == STEP_RELAX) {
    a.w[oi] = wn + e.gval;
  } else {  // STEP_RESID
    const float res = e.cur - wn - e.gval;
    const long long ai = (ro.a & ~1LL) + j;
    a.gc[ai] = -res;
    a.wc[ai] = (ro.a & 1) ? -res : 0.f;                // zero guess; -r at the marked points
    nrm += (double)res * (double)res;
  }
}

// Epilogue of one MFMA tile over the staged sums (see EpiStage).
struct AdjEpiIn4 {
  floatx4 kd, wv, gval, cur;
};
template <class C, int MODE>
__device__ inline void adj_tile_epilogue(const AdjArgs& a, Acc<C>& acc, const AdjRow* rowtab,
                                         float* stage, long long m0, int n0, long long R,
                                         double& nrm) {
  typedef EpiStage<C> E;
  const int H = a.H;
  const int c4 = E::col4();
  const int j = n0 + c4 * 4;
  const bool colok = E::active() && j < H;
  const int jc = colok ? j : H - 4;                     // clamped columns are never stored
#pragma unroll
  for (int ba = 0; ba < C::BM; ++ba) {
    __syncthreads();                                    // staging area no longer read
    E::write(acc, ba, stage);
    AdjEpiIn4 in[E::ITEMS];
    long long oo[E::ITEMS], oa[E::ITEMS];
    int trow[E::ITEMS];
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      trow[it] = E::tile_row(E::staged_row(it), ba);
      const AdjRow ro = rowtab[trow[it]];               // rows beyond the launch hold its last row
      oo[it] = ro.o;
      oa[it] = ro.a;
      in[it].kd = ldg4(a.kap + ro.k + 3 * H + jc);
      in[it].wv = ldg4(a.w_in + ro.in + jc);
      in[it].gval = a.g ? ldg4(a.g + ro.o + jc) : zero4();
      in[it].cur = MODE == STEP_RESID ? ldg4(a.w + ro.o + jc) : zero4();
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      const floatx4 dot = E::read(stage, 0, E::staged_row(it), c4);
      if (!colok || m0 + trow[it] >= R) continue;
      const floatx4 wn = in[it].kd * in[it].wv + dot;
      const long long oi = oo[it] + j;
      if (MODE == STEP_RELAX) {
        *reinterpret_cast<floatx4*>(a.w + oi) = wn + in[it].gval;
      } else {  // STEP_RESID
        const floatx4 res = in[it].cur - wn - in[it].gval;
        const long long ai = (oa[it] & ~1LL) + j;
        *reinterpret_cast<floatx4*>(a.gc + ai) = -res;
        // zero guess of the coarse error equation; -r at the marked points
        *reinterpret_cast<floatx4*>(a.wc + ai) = (oa[it] & 1) ? -res : zero4();
#pragma unroll
        for (int i = 0; i < 4; ++i) nrm += (double)res[i] * (double)res[i];
      }
    }
  }
}

struct KapW {
  floatx4 kap, w;
};

template <class C, int MODE>
__global__ __launch_bounds__(C::NT, C::MINWG) void adj_step_kernel(AdjArgs a) {
  constexpr int LDSF =
      C::LDS_FLOATS > EpiStage<C>::FLOATS ? C::LDS_FLOATS : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float lds[LDSF];
  const int H = a.H, B = a.B, K = 3 * a.H;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  __shared__ AdjRow rowtab[C::TM];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = adj_row(a, r);
  }
  // (visible to all waves after the barriers inside the contraction)

  const float* krow[C::A_CHUNKS];
  const float* wrow[C::A_CHUNKS];
  const float* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row<C>(s);
    if (r >= R) r = R - 1;     // clamped rows are never stored
    const long long pt = (unsigned)r / (unsigned)B;   // rows < 2^31: 32-bit division
    const int b = (int)(r - pt * B);
    krow[s] = a.kap + (a.k.at(pt) * B + b) * (long long)a.kw;
    wrow[s] = a.w_in + (a.in.at(pt) * B + b) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int j = n0 + chunk_row<C>(s);
    if (j >= H) j = H - 1;
    brow[s] = (const float*)a.UT + (long long)j * K;
  }
  Acc<C> acc;
  acc.zero();
  // A operand: kappa and w stay raw in registers during the MFMAs of the current
  // slice and are multiplied when the slice is written to LDS
  auto la = [&](int s, int k) {
    const int kk = k >= 2 * H ? k - 2 * H : (k >= H ? k - H : k);
    return KapW{ldg4(krow[s] + k), ldg4(wrow[s] + kk)};
  };
  auto lb = [&](int s, int k) { return ldg4(brow[s] + k); };
  auto fa = [](const KapW& r) { return r.kap * r.w; };
  if (K % C::TK == 0 && C::KS == 1 && C::BM * C::BN >= 4) {
    // Whole slices per gate (H is a multiple of the slice width): the sum over k may run
    // in any slice order, so slice i takes gate i % 3 and the columns of slice i / 3 of
    // that gate.  The three slices that multiply the same columns of w then follow each
    // other, and w is loaded for the first of them only.
    floatx4 wkeep[C::A_CHUNKS];
    auto col = [&](int k, int& kk) {
      const int i = k / C::TK;
      const int g = i % 3;
      kk = (i / 3) * C::TK + (k - i * C::TK);
      return g;
    };
    auto lag = [&](int s, int k) {
      int kk;
      const int g = col(k, kk);
      if (g == 0) wkeep[s] = ldg4(wrow[s] + kk);
      return KapW{ldg4(krow[s] + g * H + kk), wkeep[s]};
    };
    auto lbg = [&](int s, int k) {
      int kk;
      const int g = col(k, kk);
      return ldg4(brow[s] + g * H + kk);
    };
    gemm_nt_tile<C, false>(acc, K, lag, lbg, fa, Identity4(), lds);
  } else if (K % C::TK == 0) {
    gemm_nt_tile<C, false>(acc, K, la, lb, fa, Identity4(), lds);
  } else {
    gemm_nt_tile<C, true>(acc, K, la, lb, fa, Identity4(), lds);
  }

  double nrm = 0.0;
  adj_tile_epilogue<C, MODE>(a, acc, rowtab, lds, m0, n0, R, nrm);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// bf16 weights: the fp32 products kappa*w go to LDS as one bf16 tile or as hi + lo tiles
// (the configuration's A2, see gemm_core_bf16.h).
struct KapW8 {
  floatx4 k0, k1, w0, w1;
};

template <class C, int MODE>
__global__ __launch_bounds__(C::NT, C::MINWG) void adj_step_kernel_bf16(AdjArgs a) {
  constexpr int LDSF = C::LDS_ELEMS / 2 + 1 > EpiStage<C>::FLOATS ? C::LDS_ELEMS / 2 + 1
                                                                  : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float ldsf[LDSF];
  bf16_t* lds = reinterpret_cast<bf16_t*>(ldsf);
  const int H = a.H, B = a.B, K = 3 * a.H;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  const bf16_t* UT = (const bf16_t*)(C::NP == 3 ? a.UT3 : a.UT);
  __shared__ AdjRow rowtab[C::TM];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = adj_row(a, r);
  }
  // (visible to all waves after the barriers inside the contraction)

  const float* krow[C::A_CHUNKS];
  const float* wrow[C::A_CHUNKS];
  const bf16_t* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row_b<C>(s);
    if (r >= R) r = R - 1;
    const long long pt = (unsigned)r / (unsigned)B;   // rows < 2^31: 32-bit division
    const int b = (int)(r - pt * B);
    krow[s] = a.kap + (a.k.at(pt) * B + b) * (long long)a.kw;
    wrow[s] = a.w_in + (a.in.at(pt) * B + b) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int j = n0 + chunk_row_b<C>(s);
    if (j >= H) j = H - 1;
    brow[s] = UT + (long long)j * K;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) {
    const int kk = k >= 2 * H ? k - 2 * H : (k >= H ? k - H : k);
    return KapW8{ldg4(krow[s] + k), ldg4(krow[s] + k + 4), ldg4(wrow[s] + kk),
                 ldg4(wrow[s] + kk + 4)};
  };
  auto fa = [](const KapW8& r) { return F32x8{r.k0 * r.w0, r.k1 * r.w1}; };
  if constexpr (C::NP == 3) {
    const long long term = (long long)H * K;
    auto lb = [&](int s, int k) {
      return Bf16x8x3{{ldg8h(brow[s] + k), ldg8h(brow[s] + term + k),
                       ldg8h(brow[s] + 2 * term + k)}};
    };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  } else {
    auto lb = [&](int s, int k) { return ldg8h(brow[s] + k); };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  }

  double nrm = 0.0;
  adj_tile_epilogue<C, MODE>(a, acc, rowtab, ldsf, m0, n0, R, nrm);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// ---------------------------------------------------------------------------
// Input gradients: dx[R, D] = S_x[R, 3H] . WT[D, 3H]^T,  S_x = (k_r w, k_z w, k_n w)
// of step t in row (t-1)*B + b  (input-side counterpart of Alg. 3's gradient line)
// ---------------------------------------------------------------------------
typedef TileCfg<2, 2, 2, 2, 1> DxCfg;            // 128 x 128 tile
typedef TileCfgB<2, 2, 2, 2, 1, true> DxCfgB;
typedef TileCfgB<2, 2, 2, 2, 1, true, 1, 1, 2, 1, 64, false> DxCfgF;   // kappa * w as one bf16 term
typedef TileCfgB<4, 2, 1, 2, 1, true, 1, 1, 2, 3, 32> DxCfgS;     // 8 waves of 32 x 64

// Stores one accumulator tile of a plain GEMM: out[m, n], leading dimension N.
template <class C>
__device__ inline void store_tile(const Acc<C>& acc, float* out, long long m0, int n0,
                                  long long M, int N) {
#pragma unroll
  for (int a = 0; a < C::BM; ++a)
#pragma unroll
    for (int b = 0; b < C::BN; ++b) {
      int row, col;
      acc_coord<C>(a, b, 0, row, col);
      const int n = n0 + col;
      if (n >= N) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc_coord<C>(a, b, e, row, col);
        const long long m = m0 + row;
        if (m < M) out[m * N + n] = acc.v[0][a][b][e];
      }
    }
}

__global__ __launch_bounds__(DxCfg::NT) void input_grad_kernel(
    const float* __restrict__ kap0, const float* __restrict__ w, const float* __restrict__ WT,
    float* __restrict__ dx, long long R, int B, int H, int D) {
  typedef DxCfg C;
  __shared__ __attribute__((aligned(16))) float lds[C::LDS_FLOATS];
  const int K = 3 * H;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  // coefficient and adjoint rows are one time point ahead of the dx row
  const float* krow[C::A_CHUNKS];
  const float* wrow[C::A_CHUNKS];
  const float* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row<C>(s);
    if (r >= R) r = R - 1;     // clamped rows are never stored
    krow[s] = kap0 + (r + B) * (5LL * H);
    wrow[s] = w + (r + B) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int n = n0 + chunk_row<C>(s);
    if (n >= D) n = D - 1;
    brow[s] = WT + (long long)n * K;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) {
    // third gate: k_n is the fifth coefficient block
    const int kk = k >= 2 * H ? k - 2 * H : (k >= H ? k - H : k);
    const int ks = k >= 2 * H ? k + 2 * H : k;
    return KapW{ldg4(krow[s] + ks), ldg4(wrow[s] + kk)};
  };
  auto lb = [&](int s, int k) { return ldg4(brow[s] + k); };
  auto fa = [](const KapW& r) { return r.kap * r.w; };
  if (K % C::TK == 0)
    gemm_nt_tile<C, false>(acc, K, la, lb, fa, Identity4(), lds);
  else
    gemm_nt_tile<C, true>(acc, K, la, lb, fa, Identity4(), lds);
  store_tile<C>(acc, dx, m0, n0, R, D);
}

template <class C>
__global__ __launch_bounds__(C::NT, C::NT > 256 ? 2 : 1) void input_grad_kernel_bf16(
    const float* __restrict__ kap0, const float* __restrict__ w, const bf16_t* __restrict__ WT,
    float* __restrict__ dx, long long R, int B, int H, int D) {
  __shared__ __attribute__((aligned(16))) bf16_t lds[C::LDS_ELEMS];
  const int K = 3 * H;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const float* krow[C::A_CHUNKS];
  const float* wrow[C::A_CHUNKS];
  const bf16_t* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row_b<C>(s);
    if (r >= R) r = R - 1;
    krow[s] = kap0 + (r + B) * (5LL * H);
    wrow[s] = w + (r + B) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int n = n0 + chunk_row_b<C>(s);
    if (n >= D) n = D - 1;
    brow[s] = WT + (long long)n * K;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) {
    const int kk = k >= 2 * H ? k - 2 * H : (k >= H ? k - H : k);
    const int ks = k >= 2 * H ? k + 2 * H : k;
    return KapW8{ldg4(krow[s] + ks), ldg4(krow[s] + ks + 4), ldg4(wrow[s] + kk),
                 ldg4(wrow[s] + kk + 4)};
  };
  auto fa = [](const KapW8& r) { return F32x8{r.k0 * r.w0, r.k1 * r.w1}; };
  if constexpr (C::NP == 3) {
    const long long term = (long long)D * K;
    auto lb = [&](int s, int k) {
      return Bf16x8x3{{ldg8h(brow[s] + k), ldg8h(brow[s] + term + k),
                       ldg8h(brow[s] + 2 * term + k)}};
    };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  } else {
    auto lb = [&](int s, int k) { return ldg8h(brow[s] + k); };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  }
  store_tile<C>(acc, dx, m0, n0, R, D);
}

hipError_t launch_input_grads(const float* kap0, const float* w, const void* WT, float* dx, int T,
                              int B, int D, int H, int bf16, int one_term, hipStream_t s) {
  const long long R = (long long)T * B;
  prof_begin(6, s);
  if (bf16 == 2) {
    typedef DxCfgS C;
    dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(input_grad_kernel_bf16<C>, grid, dim3(C::NT), 0, s, kap0, w,
                       (const bf16_t*)WT, dx, R, B, H, D);
  } else if (bf16 && one_term) {
    typedef DxCfgF C;
    dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(input_grad_kernel_bf16<C>, grid, dim3(C::NT), 0, s, kap0, w,
                       (const bf16_t*)WT, dx, R, B, H, D);
  } else if (bf16) {
    typedef DxCfgB C;
    dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(input_grad_kernel_bf16<C>, grid, dim3(C::NT), 0, s, kap0, w,
                       (const bf16_t*)WT, dx, R, B, H, D);
  } else {
    typedef DxCfg C;
    dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (D + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(input_grad_kernel, grid, dim3(C::NT), 0, s, kap0, w, (const float*)WT, dx,
                       R, B, H, D);
  }
  prof_end(6, 2.0 * (double)R * 3 * H * D,
           4.0 * (double)R * (4.0 * H + D) + (bf16 == 1 ? 2.0 : 4.0) * 3.0 * H * D, s);
  return hipGetLastError();
}

// Few-row variant (coarsest-level solve, serial BPTT): see skinny.h
template <int CT>
struct AdjSkMaxNT {
  static constexpr int value = CT >= 8 ? 512 : SK_MAXNT;
};

template <int CT, int MODE, class WT>
__global__ __launch_bounds__(AdjSkMaxNT<CT>::value) void adj_skinny_kernel(AdjArgs a,
                                                                           int rows_block) {
  constexpr int VP = sk_pow2_ceil(SK_RR * CT);
  __shared__ float red[(SK_MAXNT / 64) * VP];
  const int H = a.H, K = 3 * a.H;
  const int R = a.nk * a.B;
  const int r0 = blockIdx.y * rows_block;
  const int rows_here = min(rows_block, R - r0);
  const SkGeom geo = sk_geom(rows_block, K);
  const int ksl = geo.ksl;
  const int tid = threadIdx.x;
  const int ks = tid & (ksl - 1), rg = tid / ksl;
  const int j0 = blockIdx.x * CT;

  const int n_out = rows_here * CT;
  const bool epi = tid < n_out && j0 + tid % CT < H;
  int e_j = 0;
  AdjRow ero = {};
  AdjEpiIn ein = {};
  if (epi) {
    ero = adj_row(a, r0 + tid / CT);
    e_j = j0 + tid % CT;
    ein = adj_epi_load<MODE>(a, ero, e_j);
  }

  // rows beyond the block are clamped to its last row (their sums are never used)
  const float* krow[SK_RR];
  const float* wrow[SK_RR];
#pragma unroll
  for (int i = 0; i < SK_RR; ++i) {
    const AdjRow ro = adj_row(a, r0 + min(rg * SK_RR + i, rows_here - 1));
    krow[i] = a.kap + ro.k;
    wrow[i] = a.w_in + ro.in;
  }
  const WT* urow[CT];
#pragma unroll
  for (int u = 0; u < CT; ++u) urow[u] = (const WT*)a.UT + (long long)min(j0 + u, H - 1) * K;
  float acc[SK_RR][CT];
  skinny_dot<CT, WT>(acc, K, ks, ksl, urow, [&](int i, int k) {
    const int kk = k >= 2 * H ? k - 2 * H : (k >= H ? k - H : k);
    return ldg4(krow[i] + k) * ldg4(wrow[i] + kk);
  });
  float v[VP];
#pragma unroll
  for (int q = 0; q < VP; ++q) v[q] = q < SK_RR * CT ? acc[q / CT][q % CT] : 0.f;
  skinny_reduce<VP>(v, red, rg, ks, ksl);
  __syncthreads();

  double nrm = 0.0;
  for (int e = tid; e < n_out; e += geo.nt) {
    const int row = e / CT, c = e % CT;
    const int j = j0 + c;
    if (j >= H) continue;
    const float dot = skinny_sum<VP>(red, row / SK_RR, (row % SK_RR) * CT + c, ksl);
    if (e == tid && epi) {
      adj_epi_finish<MODE>(a, ero, e_j, dot, ein, nrm);
    } else {   // more outputs than threads (tiny K only)
      const AdjRow ro = adj_row(a, r0 + row);
      adj_epi_finish<MODE>(a, ro, j, dot, adj_epi_load<MODE>(a, ro, j), nrm);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

typedef TileCfg<2, 2, 2, 2, 1> AdjBig;    // 128 x 128, 256 threads
typedef TileCfg<2, 2, 1, 1, 1> AdjMid;    //  64 x 64, 256 threads
typedef TileCfg<1, 1, 1, 1, 1, 128, 1, 4> AdjSmall;  //  32 x 32, 4 waves splitting K
// bf16: 8 waves of 32 x 64 each (one K-slice in flight measured 5 % faster than three with
// the register budget planned for one workgroup per CU)
typedef TileCfgB<4, 2, 1, 2, 1, true, 1, 1, 2> AdjBigB;
typedef TileCfgB<2, 2, 1, 1, 1, true> AdjMidB;
typedef TileCfgB<1, 1, 1, 1, 1, true, 4> AdjSmallB;
// the same tiles with kappa * w as one bf16 term
typedef TileCfgB<4, 2, 1, 2, 1, true, 1, 1, 2, 1, 64, false> AdjBigF;
typedef TileCfgB<2, 2, 1, 1, 1, true, 1, 1, 2, 1, 64, false> AdjMidF;
typedef TileCfgB<1, 1, 1, 1, 1, true, 4, 1, 2, 1, 64, false> AdjSmallF;
// three-term operands (K-slices of 32)
typedef TileCfgB<2, 2, 2, 2, 1, true, 1, 1, 2, 3, 32> AdjBigS;
// the same tile with 8 waves of 32 x 64 each: half the accumulators per wave, so that two
// workgroups (16 waves, 128 registers per lane) share a CU and keep twice the loads in
// flight; the relaxation mode fits that register budget, the others use the 4-wave form
typedef TileCfgB<4, 2, 1, 2, 1, true, 1, 1, 2, 3, 32> AdjBigS8;
typedef TileCfgB<2, 2, 1, 1, 1, true, 1, 1, 2, 3, 32> AdjMidS;
typedef TileCfgB<1, 1, 1, 1, 1, true, 4, 1, 2, 3, 32> AdjSmallS;

template <class C, class CB, class CS, class CF>
static void launch_adj_cfg(const AdjArgs& a, hipStream_t s) {
  const long long R = (long long)a.nk * a.B;
  dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (a.H + C::TN - 1) / C::TN));
  dim3 block(a.bf16 == 2 ? CS::NT : a.bf16 ? CB::NT : C::NT);
  static_assert(CF::TM == CB::TM && CF::TN == CB::TN && CF::NT == CB::NT, "tile shapes must agree");
  static_assert(C::TM == CB::TM && C::TN == CB::TN, "tile shapes must agree");
  static_assert(C::TM == CS::TM && C::TN == CS::TN, "tile shapes must agree");
  static_assert(AdjBigS8::TM == AdjBigS::TM && AdjBigS8::TN == AdjBigS::TN, "tile shapes must agree");
  if (a.bf16 == 2) {
    if (a.mode == STEP_RELAX && std::is_same<CS, AdjBigS>::value)
      hipLaunchKernelGGL((adj_step_kernel_bf16<AdjBigS8, STEP_RELAX>), grid, dim3(AdjBigS8::NT), 0,
                         s, a);
    else if (a.mode == STEP_RELAX)
      hipLaunchKernelGGL((adj_step_kernel_bf16<CS, STEP_RELAX>), grid, block, 0, s, a);
    else
      hipLaunchKernelGGL((adj_step_kernel_bf16<CS, STEP_RESID>), grid, block, 0, s, a);
  } else if (a.bf16 && a.one_term) {
    if (a.mode == STEP_RELAX)
      hipLaunchKernelGGL((adj_step_kernel_bf16<CF, STEP_RELAX>), grid, block, 0, s, a);
    else
      hipLaunchKernelGGL((adj_step_kernel_bf16<CF, STEP_RESID>), grid, block, 0, s, a);
  } else if (a.bf16) {
    if (a.mode == STEP_RELAX)
      hipLaunchKernelGGL((adj_step_kernel_bf16<CB, STEP_RELAX>), grid, block, 0, s, a);
    else
      hipLaunchKernelGGL((adj_step_kernel_bf16<CB, STEP_RESID>), grid, block, 0, s, a);
  } else {
    if (a.mode == STEP_RELAX)
      hipLaunchKernelGGL((adj_step_kernel<C, STEP_RELAX>), grid, block, 0, s, a);
    else
      hipLaunchKernelGGL((adj_step_kernel<C, STEP_RESID>), grid, block, 0, s, a);
  }
}

// Rows per workgroup of the few-row adjoint step: every workgroup streams the
// coefficient and adjoint rows of its row block (24H bytes per row), so the block is
// kept small and the workgroup takes more columns instead.
constexpr int ADJ_SK_ROWS = 8;

static int adj_sk_rows(long long R) { return R < ADJ_SK_ROWS ? (int)R : ADJ_SK_ROWS; }

template <int CT, int MODE>
static void launch_adj_skinny_mode(const AdjArgs& a, dim3 grid, hipStream_t s) {
  const int rb = adj_sk_rows((long long)a.nk * a.B);
  const dim3 block(sk_geom(rb, 3 * a.H).nt);
  if (a.bf16 == 1)
    hipLaunchKernelGGL((adj_skinny_kernel<CT, MODE, bf16_t>), grid, block, 0, s, a, rb);
  else
    hipLaunchKernelGGL((adj_skinny_kernel<CT, MODE, float>), grid, block, 0, s, a, rb);
}

template <int CT>
static void launch_adj_skinny(const AdjArgs& a, dim3 grid, hipStream_t s) {
  if (a.mode == STEP_RELAX)
    launch_adj_skinny_mode<CT, STEP_RELAX>(a, grid, s);
  else
    launch_adj_skinny_mode<CT, STEP_RESID>(a, grid, s);
}

// modes STEP_RELAX and STEP_RESID (the adjoint cycle solves its coarse equations for the
// error and needs no right-hand-side launch)
hipError_t launch_adj_step(const AdjArgs& a, hipStream_t s) {
  if (a.nk <= 0) return hipSuccess;
  if (a.mode != STEP_RELAX && a.mode != STEP_RESID) return hipErrorInvalidValue;
  const long long R = (long long)a.nk * a.B;
  auto tiles = [&](int tm, int tn) { return ((R + tm - 1) / tm) * ((a.H + tn - 1) / tn); };
  const int kind = R <= 2 * SK_MAXROWS ? 5 : 1;
  prof_begin(kind, s, R, a.mode);
  if (R <= 2 * SK_MAXROWS) {
    // up to four columns per workgroup (eight measured 1.8 us slower per step at 32 rows x 512)
    const int rb = adj_sk_rows(R);
    const int nrb = (int)((R + rb - 1) / rb);
    const long long hw = (long long)a.H * nrb;
    const int ct = hw >= 1024 ? 4 : (hw >= 512 ? 2 : 1);
    dim3 grid((unsigned)((a.H + ct - 1) / ct), (unsigned)nrb);
    if (ct == 4)
      launch_adj_skinny<4>(a, grid, s);
    else if (ct == 2)
      launch_adj_skinny<2>(a, grid, s);
    else
      launch_adj_skinny<1>(a, grid, s);
  } else if (tiles(AdjBig::TM, AdjBig::TN) >= (a.bf16 == 1 ? 256 : 384))
    launch_adj_cfg<AdjBig, AdjBigB, AdjBigS, AdjBigF>(a, s);
  else if (R > 32 && tiles(AdjMid::TM, AdjMid::TN) >= 256)
    launch_adj_cfg<AdjMid, AdjMidB, AdjMidS, AdjMidF>(a, s);
  else
    launch_adj_cfg<AdjSmall, AdjSmallB, AdjSmallS, AdjSmallF>(a, s);
  prof_end(kind, 6.0 * (double)R * a.H * a.H, 28.0 * (double)R * a.H, s);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// UT[cols, rows] = U[rows, cols]^T
// ---------------------------------------------------------------------------
template <class T>
__global__ void transpose_kernel(const T* __restrict__ U, T* __restrict__ UT, int rows, int cols) {
  __shared__ T t[32][33];
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    int r = r0 + i, c = c0 + tx;
    t[i][tx] = (r < rows && c < cols) ? U[(long long)r * cols + c] : T(0);
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) UT[(long long)c * rows + r] = t[tx][i];
  }
}

hipError_t launch_transpose(const void* U, void* UT, int rows, int cols, int bf16, hipStream_t s) {
  dim3 grid((cols + 31) / 32, (rows + 31) / 32);
  if (bf16)
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)U,
                       (bf16_t*)UT, rows, cols);
  else
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, s, (const float*)U,
                       (float*)UT, rows, cols);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Parameter gradients: dU = S^T Hprev, dW = Sx^T X, db_h = colsum S, db_i = colsum Sx
// with S[k, g*H+j] = kap0[k][g*H+j] * w[k][j] (gates r, z, q) and Sx the same
// except that its third block uses k_n (stored at 4H..5H) instead of k_q.
// Row k = (t-1)*B + b for step t = 1..T: kap0 and w rows are offset by one time
// point, Hprev = h[t-1] and X = x[t-1] are not.
// ---------------------------------------------------------------------------
constexpr int GTK = 32;            // K-slice (rows of the sum) per iteration
constexpr int GT = 128;            // output tile is GT x GT
constexpr int GLD = GT;            // LDS row stride in floats; odd rows swap their 32-column
                                   // halves pairwise (column ^ 32), which keeps the two
                                   // half-waves of an operand read on different banks

struct GradArgs {
  const float* kap0;   // [(T+1),B,5H]
  const float* w;      // [(T+1),B,H]
  const void* Bm;      // h[(T+1),B,H] (float) or x[T,B,D] (float or bf16); row k as is
  float* part;         // [splits][3H][N]
  float* bpart;        // [splits][3H] column sums of S (bias gradients), written by the first column tile
  long long Ktot;      // T*B
  long long Kper;      // rows per split (multiple of GTK)
  int B, H, N;         // N = H (dU) or D (dW)
  int third_off;       // 2H (k_q, dU) or 4H (k_n, dW)
  int mtiles, ntiles;  // output tiles along 3H and N
  int splits;          // row splits (a multiple of 8, or fewer than 8)
};

// C[m, n] = sum_k S[k, m] Bm[k, n] over this split's rows k.  Both operands are
// read with the contracted index k slowest, so an LDS slice is stored [k][m] and
// a lane reads its MFMA operand as one float per k-pair.
// 1-D grid: workgroups go round-robin over the 8 XCDs, so split z is given to XCD
// z % 8 and all output tiles of a split run on that XCD: its rows of S and Bm are
// fetched into one L2 only.
template <class BT>
__global__ __launch_bounds__(256, 3) void grad_gemm_kernel(GradArgs a) {
  __shared__ __attribute__((aligned(16))) float As[1][GTK * GLD];
  __shared__ __attribute__((aligned(16))) float Bs[1][GTK * GLD];
  const int H = a.H, N = a.N, M = 3 * a.H;
  const int tiles = a.mtiles * a.ntiles;
  int tile, z;
  if (a.splits % NXCD == 0) {
    const int j = blockIdx.x / NXCD;
    tile = j % tiles;
    z = (j / tiles) * NXCD + blockIdx.x % NXCD;
  } else {
    tile = blockIdx.x % tiles;
    z = blockIdx.x / tiles;
  }
  const int m0 = (tile % a.mtiles) * GT, n0 = (tile / a.mtiles) * GT;
  const long long kbeg = (long long)z * a.Kper;
  long long kend = kbeg + a.Kper;
  if (kend > a.Ktot) kend = a.Ktot;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lh = lane >> 5;
  const long long rowoff = a.B;   // kap0 / w rows are one time point ahead

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // each thread stages NCH float4 of A and of B per slice: slice row = q/32, col4 = q%32.
  // The column part is fixed per thread; out-of-range columns and rows are clamped
  // for the load and zeroed when the slice is written to LDS.
  constexpr int NCH = GTK * (GT / 4) / 256;
  const int c4 = tid & 31;
  const int m = m0 + c4 * 4, n = n0 + c4 * 4;
  const bool m_ok = m < M, n_ok = n < N;
  const int mc = m_ok ? m : 0, nc = n_ok ? n : 0;
  const int gate = mc / H, jcol = mc - gate * H;
  const int src = gate == 2 ? a.third_off + jcol : mc;
  floatx4 rk[NCH], rw[NCH], rb[NCH];
  // Bias gradients are the column sums of S: every thread adds up the products it stages
  // (its four columns, its rows of every slice); the eight row groups meet in LDS at the end.
  floatx4 colsum = zero4();
  auto fetch = [&](long long k0) {
#pragma unroll
    for (int s = 0; s < NCH; ++s) {
      long long k = k0 + (tid >> 5) + s * 8;
      if (k >= kend) k = kend - 1;
      rk[s] = ldg4(a.kap0 + (k + rowoff) * (5LL * H) + src);
      rw[s] = ldg4(a.w + (k + rowoff) * H + jcol);
      rb[s] = ldg4w((const BT*)a.Bm + k * N + nc);
    }
  };
  const int wcol = (c4 * 4) ^ (((tid >> 5) & 1) << 5);     // slice rows kr and tid >> 5: same parity
  auto stash = [&](long long k0, int buf) {
#pragma unroll
    for (int s = 0; s < NCH; ++s) {
      const int kr = (tid >> 5) + s * 8;
      const bool k_ok = k0 + kr < kend;
      const floatx4 p = (k_ok && m_ok) ? rk[s] * rw[s] : zero4();
      colsum += p;
      *reinterpret_cast<floatx4*>(&As[buf][kr * GLD + wcol]) = p;
      *reinterpret_cast<floatx4*>(&Bs[buf][kr * GLD + wcol]) = (k_ok && n_ok) ? rb[s] : zero4();
    }
  };
  auto frags = [&](int buf, int p, float (&av)[2], float (&bv)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      av[i] = As[buf][(2 * p + lh) * GLD + wm * 64 + ((i ^ lh) << 5) + li];
#pragma unroll
    for (int j = 0; j < 2; ++j)
      bv[j] = Bs[buf][(2 * p + lh) * GLD + wn * 64 + ((j ^ lh) << 5) + li];
  };

  const int nt = tile / a.mtiles;
  if (kbeg < kend) {
    fetch(kbeg);
    stash(kbeg, 0);
    __syncthreads();
    constexpr int buf = 0;
    for (long long k0 = kbeg; k0 < kend; k0 += GTK) {
      const bool more = k0 + GTK < kend;
      if (more) fetch(k0 + GTK);
      __builtin_amdgcn_sched_barrier(0);
      float av[2][2], bv[2][2];
      __builtin_amdgcn_s_setprio(2);      // MFMA phase first at issue (see gemm_core.h)
      frags(buf, 0, av[0], bv[0]);
#pragma unroll
      for (int p = 0; p < GTK / 2; ++p) {
        if (p + 1 < GTK / 2) frags(buf, p + 1, av[(p + 1) & 1], bv[(p + 1) & 1]);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[p & 1][i], bv[p & 1][j],
                                                             acc[i][j], 0, 0, 0);
        if (p + 1 < GTK / 2) {
          // one LDS read of the next k-pair, one MFMA of this pair, four times
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      if (more) {
        stash(k0 + GTK, buf);
        __syncthreads();
      }
    }
  }
  {
    float* red = As[0];                    // [8][GT] floats (the slices are no longer read)
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e) red[(tid >> 5) * GT + c4 * 4 + e] = colsum[e];
    __syncthreads();
    if (tid < GT && m0 + tid < M) {
      float sum = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) sum += red[q * GT + tid];
      // every column tile holds the same sums: the first one reports them
      if (nt == 0) a.bpart[(long long)z * M + m0 + tid] = sum;
    }
  }
  float* out = a.part + (long long)z * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int mm = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * lh + (e & 3);
        const int nn = n0 + wn * 64 + j * 32 + li;
        if (mm < M && nn < N) out[(long long)mm * N + nn] = acc[i][j][e];
      }
}

// The same contraction for the bf16-input variant on the bf16 MFMA
// (v_mfma_f32_32x32x16_bf16).  The instruction wants eight consecutive k per lane,
// the operands have k as the slow index, so the transposition happens in registers on
// the way to LDS: a thread loads an 8 (k) x 4 (m) block of kappa and w, forms the
// products and writes, for each of its four m, the eight k as one 16-byte row segment
// of a [m][k] tile - after which fragments are read exactly as in the NT kernels.
// fp32 operands (S = kappa*w, and h for dU) go to LDS as hi + lo bf16 tiles:
//   dW: S_hi x + S_lo x (x is bf16 already);  dU: S_hi h_hi + S_lo h_hi + S_hi h_lo.
// Bias gradients: column sums of the fp32 products, accumulated by the staging threads.
constexpr int HB_TK = 64;                 // k rows per slice
constexpr int HB_LD = HB_TK + 8;          // LDS row stride in bf16 elements
template <bool B_BF16>
__global__ __launch_bounds__(256, 2) void grad_gemm_bf16_kernel(GradArgs a) {
  constexpr int NBT = B_BF16 ? 1 : 2;     // B tiles in LDS (hi, lo)
  __shared__ __attribute__((aligned(16))) bf16_t As[2][GT * HB_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[NBT][GT * HB_LD];
  const int H = a.H, N = a.N, M = 3 * a.H;
  const int tiles = a.mtiles * a.ntiles;
  int tile, z;
  if (a.splits % NXCD == 0) {
    const int j = blockIdx.x / NXCD;
    tile = j % tiles;
    z = (j / tiles) * NXCD + blockIdx.x % NXCD;
  } else {
    tile = blockIdx.x % tiles;
    z = blockIdx.x / tiles;
  }
  const int nt = tile / a.mtiles;
  const int m0 = (tile % a.mtiles) * GT, n0 = nt * GT;
  const long long kbeg = (long long)z * a.Kper;
  long long kend = kbeg + a.Kper;
  if (kend > a.Ktot) kend = a.Ktot;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lh = lane >> 5;
  const long long rowoff = a.B;           // kap0 / w rows are one time point ahead

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // staging block of this thread: A: columns m4*4..+3, rows k8*8..+7 of the slice
  const int m4 = tid & 31, k8 = tid >> 5;
  const int m = m0 + m4 * 4;
  const bool m_ok = m < M;
  const int mc = m_ok ? m : 0;
  const int gate = mc / H, jcol = mc - gate * H;
  const int src = gate == 2 ? a.third_off + jcol : mc;
  // B (bf16): columns n8*8..+7, rows kb*8..+7, threads 0..127;  B (fp32): as A
  const int n8 = tid & 15, kb = B_BF16 ? (tid >> 4) : k8;
  const bool b_thread = !B_BF16 || tid < 128;
  const int n = n0 + (B_BF16 ? n8 * 8 : m4 * 4);
  const bool n_ok = n < N;
  const int nc = n_ok ? n : 0;

  // LDS chunk positions.  A thread's rows are four (fp32 operands) or eight (bf16 second
  // operand) apart, 64 or 128 bytes modulo the 256 the banks span, so the 16-byte chunk it
  // writes is exchanged with another chunk of the row, chosen by the column block (bits 4-5,
  // or 4-6, of the row; the readers apply the same exchange): sixteen neighbouring lanes
  // then cover all banks once.
  const int ka = (k8 ^ ((m4 >> 2) & 3)) * 8;              // k8 == kb for fp32 operands
  const int kbs = (kb ^ ((n8 >> 1) & 7)) * 8;
  floatx4 rk[8], rw[8];
  floatx4 rbf[B_BF16 ? 1 : 8];
  bf16x8 rbh[B_BF16 ? 8 : 1];
  float colsum[4] = {0.f, 0.f, 0.f, 0.f};
  auto fetch = [&](long long k0) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      long long k = k0 + k8 * 8 + r;
      if (k >= kend) k = kend - 1;
      rk[r] = ldg4(a.kap0 + (k + rowoff) * (5LL * H) + src);
      rw[r] = ldg4(a.w + (k + rowoff) * H + jcol);
    }
    if (b_thread) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        long long k = k0 + kb * 8 + r;
        if (k >= kend) k = kend - 1;
        if constexpr (B_BF16)
          rbh[r] = ldg8h((const bf16_t*)a.Bm + k * N + nc);
        else
          rbf[r] = ldg4((const float*)a.Bm + k * N + nc);
      }
    }
  };
  auto stash = [&](long long k0) {
    floatx4 p[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const bool k_ok = k0 + k8 * 8 + r < kend;
      p[r] = (k_ok && m_ok) ? rk[r] * rw[r] : zero4();
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      F32x8 v;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        v.lo4[r] = p[r][e];
        v.hi4[r] = p[4 + r][e];
        colsum[e] += p[r][e] + p[4 + r][e];
      }
      bf16x8 hi, lo;
      split_bf16(v, hi, lo);
      *reinterpret_cast<bf16x8*>(&As[0][(m4 * 4 + e) * HB_LD + ka]) = hi;
      *reinterpret_cast<bf16x8*>(&As[1][(m4 * 4 + e) * HB_LD + ka]) = lo;
    }
    if (b_thread) {
      if constexpr (B_BF16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          bf16x8 o;
#pragma unroll
          for (int r = 0; r < 8; ++r) {
            const bool k_ok = k0 + kb * 8 + r < kend;
            o[r] = (k_ok && n_ok) ? rbh[r][e] : (__bf16)0.f;
          }
          *reinterpret_cast<bf16x8*>(&Bs[0][(n8 * 8 + e) * HB_LD + kbs]) = o;
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          F32x8 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            v.lo4[r] = (k0 + kb * 8 + r < kend && n_ok) ? rbf[r][e] : 0.f;
            v.hi4[r] = (k0 + kb * 8 + 4 + r < kend && n_ok) ? rbf[4 + r][e] : 0.f;
          }
          bf16x8 hi, lo;
          split_bf16(v, hi, lo);
          *reinterpret_cast<bf16x8*>(&Bs[0][(m4 * 4 + e) * HB_LD + ka]) = hi;
          *reinterpret_cast<bf16x8*>(&Bs[NBT - 1][(m4 * 4 + e) * HB_LD + ka]) = lo;
        }
      }
    }
  };

  if (kbeg < kend) {
    fetch(kbeg);
    stash(kbeg);
    __syncthreads();
    for (long long k0 = kbeg; k0 < kend; k0 += HB_TK) {
      const bool more = k0 + HB_TK < kend;
      if (more) fetch(k0 + HB_TK);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int c = 0; c < HB_TK / 16; ++c) {
        bf16x8 fa[2][2], fb[NBT][2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 2; ++i)
            fa[t][i] = *reinterpret_cast<const bf16x8*>(
                &As[t][(wm * 64 + i * 32 + li) * HB_LD + ((2 * c + lh) ^ ((2 * i + (li >> 4)) & 3)) * 8]);
#pragma unroll
        for (int t = 0; t < NBT; ++t)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const int sw = B_BF16 ? (4 * wn + 2 * j + (li >> 4)) & 7 : (2 * j + (li >> 4)) & 3;
            fb[t][j] = *reinterpret_cast<const bf16x8*>(
                &Bs[t][(wn * 64 + j * 32 + li) * HB_LD + ((2 * c + lh) ^ sw) * 8]);
          }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][i], fb[0][j], acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[1][i], fb[0][j], acc[i][j], 0, 0, 0);
            if constexpr (!B_BF16)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][i], fb[NBT - 1][j], acc[i][j], 0, 0, 0);
          }
      }
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      if (more) {
        stash(k0 + HB_TK);
        __syncthreads();
      }
    }
  }
  // column sums: the eight row groups of a column meet in LDS (the A tiles are free now)
  float* red = reinterpret_cast<float*>(&As[0][0]);      // [8][GT] floats = 4 KB
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 4; ++e) red[k8 * GT + m4 * 4 + e] = colsum[e];
  __syncthreads();
  if (tid < GT && m0 + tid < M) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) sum += red[q * GT + tid];
    // every column tile holds the same sums: the first one reports them
    if (nt == 0) a.bpart[(long long)z * M + m0 + tid] = sum;
  }
  float* out = a.part + (long long)z * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int mm = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * lh + (e & 3);
        const int nn = n0 + wn * 64 + j * 32 + li;
        if (mm < M && nn < N) out[(long long)mm * N + nn] = acc[i][j][e];
      }
}

// Wide-tile form of the bf16 contraction above (128 x 256 outputs per workgroup, each wave 64 x 128),
// used when the second operand has more than 128 columns.  The kernel above is bound by the bytes
// it pulls through the vector-memory path (8 bytes of kappa and w per S element, re-read by every
// column tile); twice the columns per tile take 40 % off those.  Both operands are written to LDS
// in the order they have in memory, [k][column] (S after the product and the hi/lo split, eight
// bytes per thread and row; the second operand as loaded), and the k-major MFMA fragments are
// formed by the LDS transpose read (ds_read_b64_tr_b16): within 16 lanes, lane i receives element
// i % 4 of what lanes 4e + i / 4 (e = 0..3) point at.  With lanes 4r..4r+3 of a block pointing at
// sixteen consecutive columns of row k + r, lane i therefore gets column i of rows k..k+3; two
// reads give the eight k of a 32x32x16 operand.  Row strides are 64 bytes modulo 256, so the four
// rows of a read fall on different banks; the writes are contiguous.
constexpr int TR_TK = 32;                  // k rows per slice
constexpr int TR_GN = 256;                 // tile columns (second operand)
constexpr int TR_LDA = GT + 32;            // row strides in elements: 320 and 576 bytes
constexpr int TR_LDB = TR_GN + 32;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// eight k (rows p .. p + 7 of the LDS tile, in the lane's own order) of this lane's column
__device__ inline bf16x8 lds_tr8(const bf16_t* p, int ld) {
  typedef __attribute__((address_space(3))) short4v* lptr;
  const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)p);
  const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 4 * ld));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ inline void split_bf16_4(const floatx4& v, bf16x4& hi, bf16x4& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = (__bf16)v[i];
    lo[i] = (__bf16)(v[i] - (float)hi[i]);
  }
}

// ONE: S and an fp32 second operand enter as one bf16 term each (dtype MGRIT_BF16); otherwise as
// hi + lo, with the products S_hi B_hi + S_lo B_hi (+ S_hi B_lo for an fp32 second operand).
template <bool B_BF16, bool ONE>
__global__ __launch_bounds__(256, 2) void grad_gemm_tr_kernel(GradArgs a) {
  constexpr int NBT = (B_BF16 || ONE) ? 1 : 2;     // tiles of the second operand in LDS (hi, lo)
  constexpr int NAT = ONE ? 1 : 2;                 // tiles of S
  __shared__ __attribute__((aligned(16))) bf16_t As[NAT][TR_TK * TR_LDA];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[NBT][TR_TK * TR_LDB];
  const int H = a.H, N = a.N, M = 3 * a.H;
  const int tiles = a.mtiles * a.ntiles;
  int tile, z;
  if (a.splits % NXCD == 0) {
    const int j = blockIdx.x / NXCD;
    tile = j % tiles;
    z = (j / tiles) * NXCD + blockIdx.x % NXCD;
  } else {
    tile = blockIdx.x % tiles;
    z = blockIdx.x / tiles;
  }
  const int nt = tile / a.mtiles;
  const int m0 = (tile % a.mtiles) * GT, n0 = nt * TR_GN;
  const long long kbeg = (long long)z * a.Kper;
  long long kend = kbeg + a.Kper;
  if (kend > a.Ktot) kend = a.Ktot;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lh = lane >> 5;
  const long long rowoff = a.B;           // kap0 / w rows are one time point ahead

  floatx16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // staging of S: columns m4*4..+3, slice rows k8 + 8r (r = 0..3)
  const int m4 = tid & 31, k8 = tid >> 5;
  const int m = m0 + m4 * 4;
  const bool m_ok = m < M;
  const int mc = m_ok ? m : 0;
  const int gate = mc / H, jcol = mc - gate * H;
  const int src = gate == 2 ? a.third_off + jcol : mc;
  // second operand: bf16: columns m4*8..+7, rows k8 + 8r (r = 0..3);
  //                 fp32: columns c4*4..+3, rows kf + 4r (r = 0..7)
  const int c4 = tid & 63, kf = tid >> 6;
  const int n = n0 + (B_BF16 ? m4 * 8 : c4 * 4);
  const bool n_ok = n < N;
  const int nc = n_ok ? n : 0;
  floatx4 rk[4], rw[4];
  floatx4 rbf[B_BF16 ? 1 : 8];
  bf16x8 rbh[B_BF16 ? 4 : 1];
  floatx4 colsum = zero4();
  auto fetch = [&](long long k0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      long long k = k0 + k8 + 8 * r;
      if (k >= kend) k = kend - 1;
      rk[r] = ldg4(a.kap0 + (k + rowoff) * (5LL * H) + src);
      rw[r] = ldg4(a.w + (k + rowoff) * H + jcol);
      if constexpr (B_BF16) rbh[r] = ldg8h((const bf16_t*)a.Bm + k * N + nc);
    }
    if constexpr (!B_BF16) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        long long k = k0 + kf + 4 * r;
        if (k >= kend) k = kend - 1;
        rbf[r] = ldg4((const float*)a.Bm + k * N + nc);
      }
    }
  };
  auto stash = [&](long long k0) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = k8 + 8 * r;
      const bool k_ok = k0 + row < kend;
      const floatx4 p = (k_ok && m_ok) ? rk[r] * rw[r] : zero4();
      colsum += p;
      bf16x4 hi, lo;
      split_bf16_4(p, hi, lo);
      *reinterpret_cast<bf16x4*>(&As[0][row * TR_LDA + m4 * 4]) = hi;
      if constexpr (!ONE) *reinterpret_cast<bf16x4*>(&As[NAT - 1][row * TR_LDA + m4 * 4]) = lo;
      if constexpr (B_BF16) {
        bf16x8 zv;
#pragma unroll
        for (int i = 0; i < 8; ++i) zv[i] = (__bf16)0.f;
        *reinterpret_cast<bf16x8*>(&Bs[0][row * TR_LDB + m4 * 8]) = (k_ok && n_ok) ? rbh[r] : zv;
      }
    }
    if constexpr (!B_BF16) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int row = kf + 4 * r;
        const floatx4 v = (k0 + row < kend && n_ok) ? rbf[r] : zero4();
        bf16x4 hi, lo;
        split_bf16_4(v, hi, lo);
        *reinterpret_cast<bf16x4*>(&Bs[0][row * TR_LDB + c4 * 4]) = hi;
        if constexpr (!ONE) *reinterpret_cast<bf16x4*>(&Bs[NBT - 1][row * TR_LDB + c4 * 4]) = lo;
      }
    }
  };
  // transpose reads: lane (block b = lane / 16, i = lane % 16) points at row 8 * (b / 2) + i / 4,
  // columns 16 * (b % 2) + 4 * (i % 4) .. + 3 of a 32-column block and receives column
  // 16 * (b % 2) + i = lane % 32 of rows 8 * (lane / 32) .. + 3
  const int i16 = lane & 15, half = (lane >> 4) & 1;
  const int a_off = (lh * 8 + (i16 >> 2)) * TR_LDA + wm * 64 + half * 16 + 4 * (i16 & 3);
  const int b_off = (lh * 8 + (i16 >> 2)) * TR_LDB + wn * 128 + half * 16 + 4 * (i16 & 3);

  if (kbeg < kend) {
    fetch(kbeg);
    stash(kbeg);
    __syncthreads();
    for (long long k0 = kbeg; k0 < kend; k0 += TR_TK) {
      const bool more = k0 + TR_TK < kend;
      if (more) fetch(k0 + TR_TK);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(2);
#pragma unroll
      for (int c = 0; c < TR_TK / 16; ++c) {
        bf16x8 fa[NAT][2], fb[NBT][4];
#pragma unroll
        for (int t = 0; t < NAT; ++t)
#pragma unroll
          for (int i = 0; i < 2; ++i)
            fa[t][i] = lds_tr8(&As[t][a_off + c * 16 * TR_LDA + i * 32], TR_LDA);
#pragma unroll
        for (int t = 0; t < NBT; ++t)
#pragma unroll
          for (int j = 0; j < 4; ++j)
            fb[t][j] = lds_tr8(&Bs[t][b_off + c * 16 * TR_LDB + j * 32], TR_LDB);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][i], fb[0][j], acc[i][j], 0, 0, 0);
            if constexpr (!ONE)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[NAT - 1][i], fb[0][j], acc[i][j], 0, 0, 0);
            if constexpr (!B_BF16 && !ONE)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[0][i], fb[NBT - 1][j], acc[i][j], 0, 0, 0);
          }
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      if (more) {
        stash(k0 + TR_TK);
        __syncthreads();
      }
    }
  }
  // column sums: the eight row groups of a column meet in LDS (the A tiles are free now)
  float* red = reinterpret_cast<float*>(&As[0][0]);      // [8][GT] floats = 4 KB
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 4; ++e) red[k8 * GT + m4 * 4 + e] = colsum[e];
  __syncthreads();
  if (tid < GT && m0 + tid < M) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) sum += red[q * GT + tid];
    // every column tile holds the same sums: the first one reports them
    if (nt == 0) a.bpart[(long long)z * M + m0 + tid] = sum;
  }
  float* out = a.part + (long long)z * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int mm = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * lh + (e & 3);
        const int nn = n0 + wn * 128 + j * 32 + li;
        if (mm < M && nn < N) out[(long long)mm * N + nn] = acc[i][j][e];
      }
}

// The same partial products for fp32 operands carried as three bf16 terms each (see
// gemm_core_bf16.h): S and the second operand (h or x) are split on their way to LDS and six
// of the nine term products are kept.  K-slices of 32 rows; waves 0-1 stage S (the product
// kappa * w, transposed in registers as above), waves 2-3 stage the second operand.
constexpr int HS_TK = 32;
constexpr int HS_LD = HS_TK + 8;
__global__ __launch_bounds__(256, 2) void grad_gemm_x3_kernel(GradArgs a) {
  __shared__ __attribute__((aligned(16))) bf16_t As[3][GT * HS_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[3][GT * HS_LD];
  const int H = a.H, N = a.N, M = 3 * a.H;
  const int tiles = a.mtiles * a.ntiles;
  int tile, z;
  if (a.splits % NXCD == 0) {
    const int j = blockIdx.x / NXCD;
    tile = j % tiles;
    z = (j / tiles) * NXCD + blockIdx.x % NXCD;
  } else {
    tile = blockIdx.x % tiles;
    z = blockIdx.x / tiles;
  }
  const int nt = tile / a.mtiles;
  const int m0 = (tile % a.mtiles) * GT, n0 = nt * GT;
  const long long kbeg = (long long)z * a.Kper;
  long long kend = kbeg + a.Kper;
  if (kend > a.Ktot) kend = a.Ktot;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1, li = lane & 31, lh = lane >> 5;
  const long long rowoff = a.B;           // kap0 / w rows are one time point ahead

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // staging block of a thread: columns c4*4..+3 of its operand, rows k8*8..+7 of the slice
  const bool is_a = tid < 128;             // uniform per wave
  const int c4 = tid & 31, k8 = (tid >> 5) & 3;
  const int col = (is_a ? m0 : n0) + c4 * 4;
  const bool c_ok = col < (is_a ? M : N);
  const int cc = c_ok ? col : 0;
  const int gate = cc / H, jcol = cc - gate * H;            // (A threads)
  const int src = gate == 2 ? a.third_off + jcol : cc;
  // Rows four apart are 320 bytes apart, i.e. 64 modulo the 256 bytes the banks span: the
  // 16-byte chunk a thread writes is therefore exchanged with another chunk of its rows,
  // chosen by bits 2-3 of the column block (the readers undo it with bits 4-5 of the row),
  // so that sixteen neighbouring lanes cover all banks once.
  bf16_t* dst = (is_a ? &As[0][0] : &Bs[0][0]) + (c4 * 4) * HS_LD + (k8 ^ ((c4 >> 2) & 3)) * 8;

  // first operand row k of this thread: a coefficient row (A) or a row of h / x (B)
  const float* base0 = is_a ? a.kap0 + rowoff * (5LL * H) + src : (const float*)a.Bm + cc;
  const long long stride0 = is_a ? 5LL * H : (long long)N;
  floatx4 r0[8], r1[8];
  float colsum[4] = {0.f, 0.f, 0.f, 0.f};
  auto fetch = [&](long long k0) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      long long k = k0 + k8 * 8 + r;
      if (k >= kend) k = kend - 1;
      r0[r] = ldg4(base0 + k * stride0);
      floatx4 t = zero4();
      if (is_a) t = ldg4(a.w + (k + rowoff) * H + jcol);
      r1[r] = t;
    }
  };
  auto stash = [&](long long k0) {
    floatx4 p[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const bool ok = c_ok && k0 + k8 * 8 + r < kend;
      p[r] = ok ? (is_a ? r0[r] * r1[r] : r0[r]) : zero4();
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      F32x8 v;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        v.lo4[r] = p[r][e];
        v.hi4[r] = p[4 + r][e];
        colsum[e] += p[r][e] + p[4 + r][e];
      }
      bf16x8 t0, t1, t2;
      split_bf16_3(v, t0, t1, t2);
      *reinterpret_cast<bf16x8*>(dst + e * HS_LD) = t0;
      *reinterpret_cast<bf16x8*>(dst + GT * HS_LD + e * HS_LD) = t1;
      *reinterpret_cast<bf16x8*>(dst + 2 * GT * HS_LD + e * HS_LD) = t2;
    }
  };

  if (kbeg < kend) {
    fetch(kbeg);
    stash(kbeg);
    __syncthreads();
    for (long long k0 = kbeg; k0 < kend; k0 += HS_TK) {
      const bool more = k0 + HS_TK < kend;
      if (more) fetch(k0 + HS_TK);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(2);
#pragma unroll
      for (int c = 0; c < HS_TK / 16; ++c) {
        bf16x8 fa[3][2], fb[3][2];
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const int ch = ((2 * c + lh) ^ ((2 * i + (li >> 4)) & 3)) * 8;
            fa[t][i] = *reinterpret_cast<const bf16x8*>(
                &As[t][(wm * 64 + i * 32 + li) * HS_LD + ch]);
            fb[t][i] = *reinterpret_cast<const bf16x8*>(
                &Bs[t][(wn * 64 + i * 32 + li) * HS_LD + ch]);
          }
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
          for (int u = 0; u < 3; ++u) {
            if (t + u > 2) continue;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
              for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[t][i], fb[u][j], acc[i][j],
                                                                    0, 0, 0);
          }
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(0);
      __syncthreads();
      if (more) {
        stash(k0 + HS_TK);
        __syncthreads();
      }
    }
  }
  // column sums of S: the four row groups of a column meet in LDS (the A tiles are free now)
  float* red = reinterpret_cast<float*>(&As[0][0]);      // [4][GT] floats
  __syncthreads();
  if (is_a) {
#pragma unroll
    for (int e = 0; e < 4; ++e) red[k8 * GT + c4 * 4 + e] = colsum[e];
  }
  __syncthreads();
  if (tid < GT && m0 + tid < M) {
    float sum = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) sum += red[q * GT + tid];
    // every column tile holds the same sums: the first one reports them
    if (nt == 0) a.bpart[(long long)z * M + m0 + tid] = sum;
  }
  float* out = a.part + (long long)z * M * N;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int mm = m0 + wm * 64 + i * 32 + 8 * (e / 4) + 4 * lh + (e & 3);
        const int nn = n0 + wn * 64 + j * 32 + li;
        if (mm < M && nn < N) out[(long long)mm * N + nn] = acc[i][j][e];
      }
}

__global__ void reduce_partials_kernel(const float* __restrict__ part, float* __restrict__ out,
                                       long long n, int splits) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int z = 0; z < splits; ++z) s += part[(long long)z * n + i];
  out[i] = s;
}

// Bias gradients from the column sums the two gradient GEMMs leave behind, one row per
// row split: pu[nu][3H] (columns k_r w, k_z w, k_q w) and pw[nw][3H] (k_r w, k_z w, k_n w).
// A workgroup covers 32 columns; its eight thread rows share the splits and meet in LDS.
__global__ void __launch_bounds__(256)
bias_reduce_kernel(const float* __restrict__ pu, int nu, const float* __restrict__ pw, int nw,
                   float* __restrict__ db_i, float* __restrict__ db_h, int H) {
  __shared__ float red[2][8][32];
  const int lane = threadIdx.x & 31, grp = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + lane;
  float su = 0.f, sw = 0.f;
  if (c < 3 * H) {
    for (int z = grp; z < nu; z += 8) su += pu[(long long)z * 3 * H + c];
    if (c >= 2 * H)
      for (int z = grp; z < nw; z += 8) sw += pw[(long long)z * 3 * H + c];
  }
  red[0][grp][lane] = su;
  red[1][grp][lane] = sw;
  __syncthreads();
  if (grp == 0 && c < 3 * H) {
    su = 0.f;
    sw = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      su += red[0][q][lane];
      sw += red[1][q][lane];
    }
    db_h[c] = su;
    db_i[c] = c < 2 * H ? su : sw;
  }
}

// Row splits of a gradient GEMM.  Enough workgroups for at least two per slot (256 CUs x
// the kernel's resident workgroups: three for the fp32 kernel, two for the others); a
// multiple of 8 (whole splits per XCD) unless fewer than 8 fill the slots as well, chosen
// so that the grid is close to a whole number of rounds over the slots: a partly filled
// last round costs as much time as a full one.
// Tile columns of a gradient GEMM: the bf16 contraction takes 256 where the second operand is
// wider than one 128-column tile.
static int grad_tile_n(int N, int bf16) { return bf16 == 1 && N > GT ? TR_GN : GT; }

static int grad_splits(long long Ktot, int M, int N, int bf16) {
  const int gn = grad_tile_n(N, bf16);
  const long long tiles = (long long)((M + GT - 1) / GT) * ((N + gn - 1) / gn);
  const long long slots = bf16 == 0 ? 768 : 512;
  long long maxs = (Ktot + 4 * GTK - 1) / (4 * GTK);   // at least 4 slices per split
  if (maxs > 256) maxs = 256;
  if (maxs < 1) maxs = 1;
  long long want = (2 * slots + tiles - 1) / tiles;
  if (want > maxs) want = maxs;
  auto efficiency = [&](long long sp) {
    const double rounds = (double)(tiles * sp) / (double)slots;
    return rounds / (double)(long long)(rounds + 0.999999);
  };
  long long best = want < NXCD ? want : want / NXCD * NXCD;
  double best_eff = want < NXCD ? efficiency(want) : 0.0;
  if (best_eff >= 0.97) return (int)best;
  for (long long sp = (want + NXCD - 1) / NXCD * NXCD; sp <= maxs && sp <= 4 * want; sp += NXCD) {
    const double eff = efficiency(sp);
    if (eff > best_eff + 0.02) {
      best_eff = eff;
      best = sp;
    }
    if (eff >= 0.97) break;
  }
  return (int)best;
}

size_t grad_partial_floats(int T, int B, int D, int H, int bf16) {
  const long long Ktot = (long long)T * B;
  const size_t zu = (size_t)grad_splits(Ktot, 3 * H, H, bf16);
  const size_t zw = (size_t)grad_splits(Ktot, 3 * H, D, bf16);
  const size_t su = zu * 3 * H * H, sw = zw * 3 * H * D;
  return (su > sw ? su : sw) + (zu + zw) * 3 * H;
}

hipError_t launch_param_grads(const float* kap0, const float* w, const float* h, const void* x,
                              float* dW, float* dU, float* db_i, float* db_h, float* part,
                              int T, int B, int D, int H, int bf16, int one_term, hipStream_t s) {
  const long long Ktot = (long long)T * B;
  const int M = 3 * H;
  prof_begin(3, s);
  const size_t su = (size_t)grad_splits(Ktot, M, H, bf16) * M * H;
  const size_t sw = (size_t)grad_splits(Ktot, M, D, bf16) * M * D;
  float* bpart[2];
  int nbpart[2];
  bpart[0] = part + (su > sw ? su : sw);
  for (int which = 0; which < 2; ++which) {
    GradArgs a;
    a.kap0 = kap0;
    a.w = w;
    a.Bm = which == 0 ? (const void*)h : x;
    a.N = which == 0 ? H : D;
    a.third_off = which == 0 ? 2 * H : 4 * H;
    a.part = part;
    a.Ktot = Ktot;
    a.B = B;
    a.H = H;
    const int splits = grad_splits(Ktot, M, a.N, bf16);
    long long per = (Ktot + splits - 1) / splits;
    const int slice = bf16 == 1 ? HB_TK : GTK;      // (both multiples of the 32 of bf16 = 2)
    a.Kper = (per + slice - 1) / slice * slice;
    a.mtiles = (M + GT - 1) / GT;
    const int gn = grad_tile_n(a.N, bf16);
    a.ntiles = (a.N + gn - 1) / gn;
    a.splits = splits;
    a.bpart = bpart[which];
    nbpart[which] = splits;
    if (which == 0) bpart[1] = bpart[0] + (size_t)nbpart[0] * M;
    dim3 grid((unsigned)((long long)a.mtiles * a.ntiles * splits));
    if (bf16 == 2)
      hipLaunchKernelGGL(grad_gemm_x3_kernel, grid, dim3(256), 0, s, a);
    else if (bf16 && gn == TR_GN && which == 1 && one_term)
      hipLaunchKernelGGL((grad_gemm_tr_kernel<true, true>), grid, dim3(256), 0, s, a);
    else if (bf16 && gn == TR_GN && one_term)
      hipLaunchKernelGGL((grad_gemm_tr_kernel<false, true>), grid, dim3(256), 0, s, a);
    else if (bf16 && gn == TR_GN && which == 1)
      hipLaunchKernelGGL((grad_gemm_tr_kernel<true, false>), grid, dim3(256), 0, s, a);
    else if (bf16 && gn == TR_GN)
      hipLaunchKernelGGL((grad_gemm_tr_kernel<false, false>), grid, dim3(256), 0, s, a);
    else if (bf16 && which == 1)
      hipLaunchKernelGGL(grad_gemm_bf16_kernel<true>, grid, dim3(256), 0, s, a);
    else if (bf16)
      hipLaunchKernelGGL(grad_gemm_bf16_kernel<false>, grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(grad_gemm_kernel<float>, grid, dim3(256), 0, s, a);
    const long long n = (long long)M * a.N;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       part, which == 0 ? dU : dW, n, splits);
  }
  hipLaunchKernelGGL(bias_reduce_kernel, dim3((3 * H + 31) / 32), dim3(256), 0, s, bpart[0],
                     nbpart[0], bpart[1], nbpart[1], db_i, db_h, H);
  prof_end(3, 2.0 * (double)Ktot * M * (H + D),
           4.0 * (double)Ktot * (5.0 * H + H + H + D), s);
  return hipGetLastError();
}

}  // namespace mg
