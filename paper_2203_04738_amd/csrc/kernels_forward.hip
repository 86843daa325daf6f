// Forward kernels: input projection GEMM and the fused GRU level step
// Phi_gamma(x, h) (Eq. 1 gates + Eq. 16 / Eq. 3 update) with the MGRIT epilogues
// (relaxation update of Alg. 1, residual + restriction of Alg. 2 lines 2-3, the
// right-hand side of Eq. 11, and the adjoint coefficient vectors).
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "common.h"
#include "gates.h"
#include "gemm_core.h"
#include "gemm_core_bf16.h"
#include "skinny.h"

namespace mg {

// ---------------------------------------------------------------------------
// Projection: P[M,N] = X[M,K] W[N,K]^T + bias[N]       (input half of Eq. 1)
// ---------------------------------------------------------------------------
typedef TileCfg<2, 2, 2, 2, 1> ProjCfg;   // 128 x 128 tile, 256 threads

__global__ __launch_bounds__(ProjCfg::NT) void projection_kernel(
    const float* __restrict__ X, const float* __restrict__ W, const float* __restrict__ bias,
    float* __restrict__ P, long long M, int N, int K) {
  typedef ProjCfg C;
  __shared__ __attribute__((aligned(16))) float lds[C::LDS_FLOATS];
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (M + C::TM - 1) / C::TM, (N + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;

  // rows beyond the matrix are clamped to its last row (their results are never
  // stored); k beyond K contributes zeros
  const float* arow[C::A_CHUNKS];
  const float* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row<C>(s);
    arow[s] = X + (r < M ? r : M - 1) * K;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int r = n0 + chunk_row<C>(s);
    brow[s] = W + (long long)(r < N ? r : N - 1) * K;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) { return ldg4(arow[s] + k); };
  auto lb = [&](int s, int k) { return ldg4(brow[s] + k); };
  if (K % C::TK == 0)
    gemm_nt_tile<C, false>(acc, K, la, lb, Identity4(), Identity4(), lds);
  else
    gemm_nt_tile<C, true>(acc, K, la, lb, Identity4(), Identity4(), lds);

#pragma unroll
  for (int a = 0; a < C::BM; ++a)
#pragma unroll
    for (int b = 0; b < C::BN; ++b) {
      int row, col;
      acc_coord<C>(a, b, 0, row, col);
      const int n = n0 + col;
      if (n >= N) continue;
      const float bv = bias[n];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc_coord<C>(a, b, e, row, col);
        const long long m = m0 + row;
        if (m < M) P[m * N + n] = acc.v[0][a][b][e] + bv;
      }
    }
}

// bf16 inputs and weights (ProjCfgB), or fp32 inputs with the weights given as their three
// bf16 terms W3[3][N,K] (ProjCfgS); fp32 accumulation and output
typedef TileCfgB<2, 2, 2, 2, 1, false> ProjCfgB;
typedef TileCfgB<4, 2, 1, 2, 1, true, 1, 1, 2, 3, 32> ProjCfgS;   // 8 waves of 32 x 64

template <class C>
__global__ __launch_bounds__(C::NT, C::NT > 256 ? 2 : 1) void projection_kernel_bf16(
    const void* __restrict__ Xv, const bf16_t* __restrict__ W, const float* __restrict__ bias,
    float* __restrict__ P, long long M, int N, int K) {
  typedef typename std::conditional<C::SPLIT_A, float, bf16_t>::type AT;
  const AT* X = (const AT*)Xv;
  __shared__ __attribute__((aligned(16))) bf16_t lds[C::LDS_ELEMS];
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (M + C::TM - 1) / C::TM, (N + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const AT* arow[C::A_CHUNKS];
  const bf16_t* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row_b<C>(s);
    arow[s] = X + (r < M ? r : M - 1) * K;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int r = n0 + chunk_row_b<C>(s);
    brow[s] = W + (long long)(r < N ? r : N - 1) * K;
  }
  Acc<C> acc;
  acc.zero();
  if constexpr (C::NP == 3) {
    const long long term = (long long)N * K;
    auto la = [&](int s, int k) { return F32x8{ldg4(arow[s] + k), ldg4(arow[s] + k + 4)}; };
    auto lb = [&](int s, int k) {
      return Bf16x8x3{{ldg8h(brow[s] + k), ldg8h(brow[s] + term + k),
                       ldg8h(brow[s] + 2 * term + k)}};
    };
    auto fa = [](const F32x8& v) { return v; };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  } else {
    auto la = [&](int s, int k) { return ldg8h(arow[s] + k); };
    auto lb = [&](int s, int k) { return ldg8h(brow[s] + k); };
    auto fa = [](const bf16x8& v) { return v; };
    if (K % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, K, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, K, la, lb, fa, lds);
  }
#pragma unroll
  for (int a = 0; a < C::BM; ++a)
#pragma unroll
    for (int b = 0; b < C::BN; ++b) {
      int row, col;
      acc_coord<C>(a, b, 0, row, col);
      const int n = n0 + col;
      if (n >= N) continue;
      const float bv = bias[n];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        acc_coord<C>(a, b, e, row, col);
        const long long m = m0 + row;
        if (m < M) P[m * N + n] = acc.v[0][a][b][e] + bv;
      }
    }
}

hipError_t launch_projection(const void* X, const void* W, const float* bias, float* P,
                             long long M, int N, int K, int bf16, hipStream_t s) {
  prof_begin(2, s);
  if (bf16 == 2) {
    typedef ProjCfgS C;
    dim3 grid((unsigned)xcd_grid((M + C::TM - 1) / C::TM, (N + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(projection_kernel_bf16<C>, grid, dim3(C::NT), 0, s, X, (const bf16_t*)W,
                       bias, P, M, N, K);
  } else if (bf16) {
    typedef ProjCfgB C;
    dim3 grid((unsigned)xcd_grid((M + C::TM - 1) / C::TM, (N + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(projection_kernel_bf16<C>, grid, dim3(C::NT), 0, s, X, (const bf16_t*)W,
                       bias, P, M, N, K);
  } else {
    typedef ProjCfg C;
    dim3 grid((unsigned)xcd_grid((M + C::TM - 1) / C::TM, (N + C::TN - 1) / C::TN));
    hipLaunchKernelGGL(projection_kernel, grid, dim3(C::NT), 0, s, (const float*)X,
                       (const float*)W, bias, P, M, N, K);
  }
  const double esz = bf16 == 1 ? 2.0 : 4.0;
  prof_end(2, 2.0 * (double)M * N * K, esz * ((double)M * K + (double)N * K) + 4.0 * (double)M * N,
           s);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Fused level step
// ---------------------------------------------------------------------------
// Operands of one output element that do not depend on the contraction: they are
// loaded separately so that the few-row kernel can fetch them before its dot
// products instead of after.
struct PhiEpiIn {
  float pr, pz, pn, h, gval, cur;
  float pr2, pz2, pn2, cur2;     // STEP_RELAX_RHS: projection and current value of the coarse step
  float prep;                    // STEP_RESID with resid_adds: the prepared half of the right-hand side
};
// Element offsets (column 0) of one row (level point, batch element) of a launch into
// the arrays the epilogue touches: input state, projection, out/cur/g, and the coarse
// (or coefficient) array.  Computed once per tile row and kept in LDS: the index
// arithmetic (a division by B and 64-bit products) is not repeated per element.
struct PhiRow {
  long long in, p, o, a;
};
__device__ inline PhiRow phi_row(const PhiArgs& a, long long r, int aux_width) {
  const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
  const int b = (int)(r - pt * a.B);
  PhiRow ro;
  ro.in = (a.in.at(pt) * a.B + b) * a.H;
  ro.p = (a.p.at(pt) * a.B + b) * (3LL * a.H);
  ro.o = (a.o.at(pt) * a.B + b) * a.H;
  ro.a = ((aux_width == a.H ? a.a.at(pt) : a.o.at(pt)) * a.B + b) * (long long)aux_width;
  // (row offsets are multiples of four elements: bit 0 marks the coarse points of ff_cf / ff_rem)
  if (a.ff_cf > 0 && a.a.at(pt) % a.ff_cf == a.ff_rem) ro.a |= 1;
  return ro;
}
// STEP_RELAX_KAPPA2: element offset of the row's coarse output point (index a) in the coarse
// level's coefficient array (4H wide).
__device__ inline long long phi_row_coarse_kappa(const PhiArgs& a, long long r) {
  const long long pt = (unsigned)r / (unsigned)a.B;
  const int b = (int)(r - pt * a.B);
  return (a.a.at(pt) * a.B + b) * (4LL * a.H);
}
struct PhiBias {          // recurrent biases of one hidden column
  float r, z, n;
};
__device__ inline PhiBias phi_bias_load(const PhiArgs& a, int j) {
  return PhiBias{a.b_h[j], a.b_h[a.H + j], a.b_h[2 * a.H + j]};
}

template <int MODE>
__device__ inline PhiEpiIn phi_epi_load(const PhiArgs& a, const PhiRow& ro, int j) {
  const int H = a.H;
  PhiEpiIn e;
  const float* pp = a.P + ro.p;
  e.pr = pp[j];
  e.pz = pp[H + j];
  e.pn = pp[2 * H + j];
  e.h = a.u_in[ro.in + j];
  const long long oi = ro.o + j;
  e.gval = (MODE != STEP_KAPPA && a.g) ? a.g[oi] : 0.f;
  e.cur = (MODE == STEP_RESID || MODE == STEP_RHS) ? a.u[oi] : 0.f;
  e.pr2 = e.pz2 = e.pn2 = e.cur2 = e.prep = 0.f;
  if (MODE == STEP_RELAX_RHS || MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK) {
    const float* p2 = pp + a.dp2;
    e.pr2 = p2[j];
    e.pz2 = p2[H + j];
    e.pn2 = p2[2 * H + j];
    if (MODE == STEP_RELAX_RHS) e.cur2 = a.u[oi + a.do2];
  }
  if (MODE == STEP_RESID && a.resid_adds) e.prep = a.gc[(ro.a & ~1LL) + j];
  return e;
}

// Gates of Eq. 1, the update of Eq. 16 / Eq. 3 and the mode-specific outputs of one
// element, given the three recurrent contractions (U_r h)_j, (U_z h)_j, (U_n h)_j.
//   RELAX: v0 = new state (+ g)          RESID: v0 = -r (coarse right-hand side), v1 = cur
//   RHS:   v0 = cur - step + g           KAPPA: v0..v4 = k_r, k_z, k_q, k_d, k_n
struct PhiOut {
  float v0, v1, v2, v3, v4, v5;       // v5: new state (+ g) of STEP_RELAX_KAPPA
  float c0, c1, c2, c3;               // STEP_RELAX_KAPPA2: k_r, k_z, k_q, k_d of the coarse step
};
// Coefficient vectors of the transposed Jacobian of one step (Appendix A.2), from its gates.
struct PhiKappa {
  float kr, kz, kq, kd, kn;
};
__device__ inline PhiKappa phi_kappa(float gamma, bool implicit, float h, float rg, float zg,
                                     float q, float n, float c, float rd, float hn) {
  float kd, dn, dz;
  if (implicit) {
    kd = rd;
    dn = gamma * c * rd;
    dz = -gamma * (n - hn) * rd;
  } else {
    kd = 1.0f - gamma * c;
    dn = gamma * c;
    dz = -gamma * (n - h);
  }
  const float kn = dn * (1.0f - n * n);
  return PhiKappa{kn * q * rg * (1.0f - rg), dz * zg * (1.0f - zg), kn * rg, kd, kn};
}
template <int MODE>
__device__ inline PhiOut phi_elem(float gamma, bool implicit, float sr, float sz, float sn,
                                  const PhiEpiIn& e, const PhiBias& bh, float gamma2 = 0.f) {
  const float h = e.h;
  const float rg = sigmoidf_(e.pr + sr + bh.r);
  const float zg = sigmoidf_(e.pz + sz + bh.z);
  const float q = sn + bh.n;
  const float n = tanhf_(e.pn + rg * q);
  const float c = 1.0f - zg;
  const float d = 1.0f + gamma * c;
  const float rd = fast_rcp(d);
  const float hn = implicit ? (h + gamma * c * n) * rd : h + gamma * c * (n - h);
  PhiOut o{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (MODE == STEP_RELAX_KAPPA || MODE == STEP_RELAX_KAPPA2) o.v5 = hn + e.gval;
  if (MODE == STEP_RELAX) {
    o.v0 = hn + e.gval;
  } else if (MODE == STEP_RELAX_RHS) {
    o.v0 = hn + e.gval;
    // the coarse level's step from the same state: same sums, its own projection and step size
    const float rg2 = sigmoidf_(e.pr2 + sr + bh.r);
    const float zg2 = sigmoidf_(e.pz2 + sz + bh.z);
    const float n2 = tanhf_(e.pn2 + rg2 * q);
    const float c2 = 1.0f - zg2;
    const float hn2 = implicit ? (h + gamma2 * c2 * n2) * fast_rcp(1.0f + gamma2 * c2)
                               : h + gamma2 * c2 * (n2 - h);
    o.v1 = e.cur2 - hn2;
  } else if (MODE == STEP_RELAX_CK) {
    o.v0 = hn + e.gval;
    // coefficient vectors of the coarser level's step from the same state
    const float rg2 = sigmoidf_(e.pr2 + sr + bh.r);
    const float zg2 = sigmoidf_(e.pz2 + sz + bh.z);
    const float n2 = tanhf_(e.pn2 + rg2 * q);
    const float c2 = 1.0f - zg2;
    const float rd2 = fast_rcp(1.0f + gamma2 * c2);
    const float hn2 = implicit ? (h + gamma2 * c2 * n2) * rd2 : h + gamma2 * c2 * (n2 - h);
    const PhiKappa k2 = phi_kappa(gamma2, implicit, h, rg2, zg2, q, n2, c2, rd2, hn2);
    o.c0 = k2.kr;
    o.c1 = k2.kz;
    o.c2 = k2.kq;
    o.c3 = k2.kd;
  } else if (MODE == STEP_RESID) {
    o.v0 = -(e.cur - hn - e.gval);
    o.v1 = e.cur;
  } else if (MODE == STEP_RHS) {
    o.v0 = (e.cur - hn) + e.gval;
  } else {  // STEP_KAPPA (and the relaxation modes that keep them): coefficients of this step
    const PhiKappa k = phi_kappa(gamma, implicit, h, rg, zg, q, n, c, rd, hn);
    o.v0 = k.kr;
    o.v1 = k.kz;
    o.v2 = k.kq;
    o.v3 = k.kd;
    o.v4 = k.kn;
    if (MODE == STEP_RELAX_KAPPA2) {
      // the coarse level's step from the same state: same sums, its own projection and step size
      const float rg2 = sigmoidf_(e.pr2 + sr + bh.r);
      const float zg2 = sigmoidf_(e.pz2 + sz + bh.z);
      const float n2 = tanhf_(e.pn2 + rg2 * q);
      const float c2 = 1.0f - zg2;
      const float rd2 = fast_rcp(1.0f + gamma2 * c2);
      const float hn2 = implicit ? (h + gamma2 * c2 * n2) * rd2 : h + gamma2 * c2 * (n2 - h);
      const PhiKappa k2 = phi_kappa(gamma2, implicit, h, rg2, zg2, q, n2, c2, rd2, hn2);
      o.c0 = k2.kr;
      o.c1 = k2.kz;
      o.c2 = k2.kq;
      o.c3 = k2.kd;
    }
  }
  return o;
}

// Scalar form used by the few-row kernel: computes and stores one element of row ro.
template <int MODE>
__device__ inline void phi_epi_finish(const PhiArgs& a, const PhiRow& ro, int j, float sr,
                                      float sz, float sn, const PhiEpiIn& e, const PhiBias& bh,
                                      double& nrm, long long coarse_kappa_row = 0) {
  const int H = a.H;
  const PhiOut o =
      phi_elem<MODE>(a.gamma, a.propagator == MGRIT_PROP_IMPLICIT, sr, sz, sn, e, bh, a.gamma2);
  const long long oi = ro.o + j;
  if (MODE == STEP_RELAX) {
    a.u[oi] = o.v0;
  } else if (MODE == STEP_RELAX_RHS) {
    a.u[oi] = o.v0;
    a.gc[ro.a + j] = o.v1;
  } else if (MODE == STEP_RELAX_CK) {
    a.u[oi] = o.v0;
    float* kc = a.gc + coarse_kappa_row;
    kc[j] = o.c0;
    kc[H + j] = o.c1;
    kc[2 * H + j] = o.c2;
    kc[3 * H + j] = o.c3;
  } else if (MODE == STEP_RESID) {
    const long long ai = (ro.a & ~1LL) + j;
    a.gc[ai] = a.resid_adds ? e.prep + o.v0 : o.v0;
    a.uc[ai] = (ro.a & 1) ? o.v1 + o.v0 : o.v1;        // cur - r at the marked points
    nrm += (double)o.v0 * (double)o.v0;
  } else if (MODE == STEP_RHS) {
    a.g[oi] = o.v0;
  } else {
    if (MODE == STEP_RELAX_KAPPA || MODE == STEP_RELAX_KAPPA2) a.u[oi] = o.v5;
    float* kp = a.uc + ro.a;
    kp[j] = o.v0;
    kp[H + j] = o.v1;
    kp[2 * H + j] = o.v2;
    kp[3 * H + j] = o.v3;
    if (a.kappa_width >= 5 * H) kp[4 * H + j] = o.v4;
    if (MODE == STEP_RELAX_KAPPA2) {
      float* kc = a.gc + coarse_kappa_row;
      kc[j] = o.c0;
      kc[H + j] = o.c1;
      kc[2 * H + j] = o.c2;
      kc[3 * H + j] = o.c3;
    }
  }
}

// Epilogue of one MFMA tile over the staged sums (see EpiStage): per pass a thread
// requests the operands of its items, the sums go through LDS, and each item is
// finished and stored as float4.
struct PhiEpiIn4 {
  floatx4 pr, pz, pn, h, gval, cur;
};
struct PhiEpiExtra4 {     // STEP_RELAX_RHS (pr2..cur2) and STEP_RESID with resid_adds (prep)
  floatx4 pr2, pz2, pn2, cur2, prep;
};

template <class C, int MODE>
__device__ inline void phi_tile_epilogue(const PhiArgs& a, Acc<C>& acc, const PhiRow* rowtab,
                                         float* stage, long long m0, int n0, long long R,
                                         double& nrm, const long long* rowtab2 = nullptr) {
  typedef EpiStage<C> E;
  const int H = a.H;
  const int c4 = E::col4();
  const int j = n0 + c4 * 4;
  const bool colok = E::active() && j < H;
  const int jc = colok ? j : H - 4;                     // clamped columns are never stored
  PhiBias bh[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) bh[i] = phi_bias_load(a, jc + i);
  const float gamma = a.gamma;
  const bool implicit = a.propagator == MGRIT_PROP_IMPLICIT;

#pragma unroll
  for (int ba = 0; ba < C::BM; ++ba) {
    __syncthreads();                                    // staging area no longer read
    E::write(acc, ba, stage);
    // operands that do not depend on the sums: requested before the barrier
    PhiEpiIn4 in[E::ITEMS];
    constexpr bool CK = MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK;
    constexpr bool EXTRA = MODE == STEP_RELAX_RHS || MODE == STEP_RESID || CK;
    PhiEpiExtra4 ex[EXTRA ? E::ITEMS : 1];
    long long oo[E::ITEMS], oa[E::ITEMS];
    long long oa2[CK ? E::ITEMS : 1];
    int trow[E::ITEMS];
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      trow[it] = E::tile_row(E::staged_row(it), ba);
      const PhiRow ro = rowtab[trow[it]];               // rows beyond the launch hold its last row
      oo[it] = ro.o;
      oa[it] = ro.a;
      const float* pp = a.P + ro.p + jc;
      in[it].pr = ldg4_stream(pp);
      in[it].pz = ldg4_stream(pp + H);
      in[it].pn = ldg4_stream(pp + 2 * H);
      in[it].h = ldg4(a.u_in + ro.in + jc);
      if (MODE != STEP_KAPPA && a.g) in[it].gval = ldg4(a.g + ro.o + jc);
      else in[it].gval = zero4();
      if (MODE == STEP_RESID || MODE == STEP_RHS) in[it].cur = ldg4(a.u + ro.o + jc);
      else in[it].cur = zero4();
      if (MODE == STEP_RELAX_RHS || CK) {
        ex[it].pr2 = ldg4_stream(pp + a.dp2);
        ex[it].pz2 = ldg4_stream(pp + a.dp2 + H);
        ex[it].pn2 = ldg4_stream(pp + a.dp2 + 2 * H);
        if (MODE == STEP_RELAX_RHS) ex[it].cur2 = ldg4(a.u + ro.o + a.do2 + jc);
        if (CK) oa2[it] = rowtab2[trow[it]];
      }
      if (MODE == STEP_RESID)
        ex[it].prep = a.resid_adds ? ldg4(a.gc + (ro.a & ~1LL) + jc) : zero4();
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      const int rp = E::staged_row(it);
      const floatx4 sr = E::read(stage, 0, rp, c4);
      const floatx4 sz = E::read(stage, 1, rp, c4);
      const floatx4 sn = E::read(stage, 2, rp, c4);
      floatx4 o0, o1, o2, o3, o4, o5;
      floatx4 q0, q1, q2, q3;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        PhiEpiIn e1{in[it].pr[i], in[it].pz[i], in[it].pn[i], in[it].h[i], in[it].gval[i],
                    in[it].cur[i], 0.f, 0.f, 0.f, 0.f, 0.f};
        if (MODE == STEP_RELAX_RHS || CK) {
          e1.pr2 = ex[it].pr2[i];
          e1.pz2 = ex[it].pz2[i];
          e1.pn2 = ex[it].pn2[i];
          if (MODE == STEP_RELAX_RHS) e1.cur2 = ex[it].cur2[i];
        }
        const PhiOut o = phi_elem<MODE>(gamma, implicit, sr[i], sz[i], sn[i], e1, bh[i], a.gamma2);
        o0[i] = o.v0; o1[i] = o.v1; o2[i] = o.v2; o3[i] = o.v3; o4[i] = o.v4; o5[i] = o.v5;
        q0[i] = o.c0; q1[i] = o.c1; q2[i] = o.c2; q3[i] = o.c3;
      }
      if (!colok || m0 + trow[it] >= R) continue;
      const long long oi = oo[it] + j;
      if (MODE == STEP_RELAX) {
        *reinterpret_cast<floatx4*>(a.u + oi) = o0;
      } else if (MODE == STEP_RELAX_RHS) {
        *reinterpret_cast<floatx4*>(a.u + oi) = o0;
        *reinterpret_cast<floatx4*>(a.gc + oa[it] + j) = o1;
      } else if (MODE == STEP_RELAX_CK) {
        *reinterpret_cast<floatx4*>(a.u + oi) = o0;
        float* kc = a.gc + oa2[it] + j;
        *reinterpret_cast<floatx4*>(kc) = q0;
        *reinterpret_cast<floatx4*>(kc + H) = q1;
        *reinterpret_cast<floatx4*>(kc + 2 * H) = q2;
        *reinterpret_cast<floatx4*>(kc + 3 * H) = q3;
      } else if (MODE == STEP_RESID) {
        const long long ai = (oa[it] & ~1LL) + j;
        // (adding the zero of a launch without a prepared half changes no value)
        *reinterpret_cast<floatx4*>(a.gc + ai) = ex[it].prep + o0;
        *reinterpret_cast<floatx4*>(a.uc + ai) = (oa[it] & 1) ? o1 + o0 : o1;   // cur - r if marked
#pragma unroll
        for (int i = 0; i < 4; ++i) nrm += (double)o0[i] * (double)o0[i];
      } else if (MODE == STEP_RHS) {
        *reinterpret_cast<floatx4*>(a.g + oi) = o0;
      } else {
        if (MODE == STEP_RELAX_KAPPA || MODE == STEP_RELAX_KAPPA2)
          *reinterpret_cast<floatx4*>(a.u + oi) = o5;
        float* kp = a.uc + oa[it] + j;
        *reinterpret_cast<floatx4*>(kp) = o0;
        *reinterpret_cast<floatx4*>(kp + H) = o1;
        *reinterpret_cast<floatx4*>(kp + 2 * H) = o2;
        *reinterpret_cast<floatx4*>(kp + 3 * H) = o3;
        if (a.kappa_width >= 5 * H) *reinterpret_cast<floatx4*>(kp + 4 * H) = o4;
        if (MODE == STEP_RELAX_KAPPA2) {
          float* kc = a.gc + oa2[it] + j;
          *reinterpret_cast<floatx4*>(kc) = q0;
          *reinterpret_cast<floatx4*>(kc + H) = q1;
          *reinterpret_cast<floatx4*>(kc + 2 * H) = q2;
          *reinterpret_cast<floatx4*>(kc + 3 * H) = q3;
        }
      }
    }
  }
}

// ZS: the launch knows that the input states of the rows from a.zero_from on are zero (its
// own instantiation, so that kernel traces list these launches apart).
template <class C, int MODE, bool ZS = false>
__global__ __launch_bounds__(C::NT, C::MINWG) void phi_step_kernel(PhiArgs a) {
  constexpr int LDSF = C::LDS_FLOATS > EpiStage<C>::FLOATS ? C::LDS_FLOATS : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float lds[LDSF];
  const int H = a.H, B = a.B;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  __shared__ PhiRow rowtab[C::TM];
  __shared__ long long rowtab2[(MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK) ? C::TM : 1];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = phi_row(a, r,
                          (MODE == STEP_KAPPA || MODE == STEP_RELAX_KAPPA ||
                           MODE == STEP_RELAX_KAPPA2) ? a.kappa_width : H);
    if (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
      rowtab2[tid] = phi_row_coarse_kappa(a, r);
  }
  // (visible to all waves after the barriers inside the contraction)

  // A rows: states of the points this tile covers (row = point*B + b); rows beyond
  // the launch are clamped to its last row and never stored.
  const float* arow[C::A_CHUNKS];
  const float* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row<C>(s);
    if (r >= R) r = R - 1;
    const long long pt = (unsigned)r / (unsigned)B;   // rows < 2^31: 32-bit division
    const int b = (int)(r - pt * B);
    arow[s] = a.u_in + (a.in.at(pt) * B + b) * H;
  }
  // B rows: for gate g the rows n0.. of U_g.
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    const int tr = chunk_row<C>(s);
    const int g = tr / C::TN;
    int j = n0 + tr % C::TN;
    if (j >= H) j = H - 1;
    brow[s] = (const float*)a.U + ((long long)g * H + j) * H;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) { return ldg4(arow[s] + k); };
  auto lb = [&](int s, int k) { return ldg4(brow[s] + k); };
  // a tile whose input states are known to be zero keeps its zero sums (uniform per workgroup)
  const bool zero_in = ZS && m0 >= a.zero_from;
  if (zero_in) {
  } else if (H % C::TK == 0)
    gemm_nt_tile<C, false>(acc, H, la, lb, Identity4(), Identity4(), lds);
  else
    gemm_nt_tile<C, true>(acc, H, la, lb, Identity4(), Identity4(), lds);

  double nrm = 0.0;
  phi_tile_epilogue<C, MODE>(a, acc, rowtab, lds, m0, n0, R, nrm, rowtab2);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// bf16 weights: the fp32 state rows go to LDS as one bf16 tile or as hi + lo tiles (the
// configuration's A2, see gemm_core_bf16.h); gates, update and outputs stay fp32.  With a three-term
// configuration the weights are fp32 values held as three bf16 arrays.
template <class C, int MODE, bool ZS = false>
__global__ __launch_bounds__(C::NT, C::MINWG) void phi_step_kernel_bf16(PhiArgs a) {
  constexpr int LDSF =
      C::LDS_ELEMS / 2 + 1 > EpiStage<C>::FLOATS ? C::LDS_ELEMS / 2 + 1 : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float ldsf[LDSF];
  bf16_t* lds = reinterpret_cast<bf16_t*>(ldsf);
  const int H = a.H, B = a.B;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  const bf16_t* U = (const bf16_t*)(C::NP == 3 ? a.U3 : a.U);
  __shared__ PhiRow rowtab[C::TM];
  __shared__ long long rowtab2[(MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK) ? C::TM : 1];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = phi_row(a, r,
                          (MODE == STEP_KAPPA || MODE == STEP_RELAX_KAPPA ||
                           MODE == STEP_RELAX_KAPPA2) ? a.kappa_width : H);
    if (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
      rowtab2[tid] = phi_row_coarse_kappa(a, r);
  }
  // (visible to all waves after the barriers inside the contraction)

  const float* arow[C::A_CHUNKS];
  const bf16_t* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row_b<C>(s);
    if (r >= R) r = R - 1;
    const long long pt = (unsigned)r / (unsigned)B;   // rows < 2^31: 32-bit division
    const int b = (int)(r - pt * B);
    arow[s] = a.u_in + (a.in.at(pt) * B + b) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    const int tr = chunk_row_b<C>(s);
    const int g = tr / C::TN;
    int j = n0 + tr % C::TN;
    if (j >= H) j = H - 1;
    brow[s] = U + ((long long)g * H + j) * H;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) { return F32x8{ldg4(arow[s] + k), ldg4(arow[s] + k + 4)}; };
  auto fa = [](const F32x8& v) { return v; };
  const bool zero_in = ZS && m0 >= a.zero_from;                // see phi_step_kernel
  if (zero_in) {
  } else if constexpr (C::NP == 3) {
    const long long term = 3LL * H * H;
    auto lb = [&](int s, int k) {
      return Bf16x8x3{{ldg8h(brow[s] + k), ldg8h(brow[s] + term + k),
                       ldg8h(brow[s] + 2 * term + k)}};
    };
    if (H % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, H, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, H, la, lb, fa, lds);
  } else {
    auto lb = [&](int s, int k) { return ldg8h(brow[s] + k); };
    if (H % C::TK == 0)
      gemm_nt_tile_bf16<C, false>(acc, H, la, lb, fa, lds);
    else
      gemm_nt_tile_bf16<C, true>(acc, H, la, lb, fa, lds);
  }

  double nrm = 0.0;
  phi_tile_epilogue<C, MODE>(a, acc, rowtab, ldsf, m0, n0, R, nrm, rowtab2);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// ---------------------------------------------------------------------------
// Few-row variant (coarsest-level propagation, serial scan): see skinny.h
// ---------------------------------------------------------------------------
// Workgroups with many columns keep RR x 3 CT sums plus their operands in registers:
// those instantiations are limited to 512 threads.
template <int CT>
struct PhiSkMaxNT {
  static constexpr int value = CT >= 4 ? 512 : SK_MAXNT;
};

template <int CT, int MODE, class WT>
__global__ __launch_bounds__(PhiSkMaxNT<CT>::value) void phi_skinny_kernel(PhiArgs a,
                                                                           int rows_block) {
  constexpr int NU = 3 * CT;
  constexpr int VP = sk_pow2_ceil(SK_RR * NU);
  __shared__ float red[(SK_MAXNT / 64) * VP];
  const int H = a.H;
  const int R = a.nk * a.B;
  const int r0 = blockIdx.y * rows_block;
  const int rows_here = min(rows_block, R - r0);
  const SkGeom geo = sk_geom(rows_block, H);
  const int ksl = geo.ksl;
  const int tid = threadIdx.x;
  const int ks = tid & (ksl - 1), rg = tid / ksl;
  const int j0 = blockIdx.x * CT;
  const int aux_w =
      (MODE == STEP_KAPPA || MODE == STEP_RELAX_KAPPA || MODE == STEP_RELAX_KAPPA2) ? a.kappa_width
                                                                                    : H;

  // this thread's output element (if any): its operands are requested first so
  // that their latency overlaps the dot products
  const int n_out = rows_here * CT;
  const bool epi = tid < n_out && j0 + tid % CT < H;
  int e_j = 0;
  PhiRow ero = {};
  PhiEpiIn ein = {};
  PhiBias ebh = {};
  if (epi) {
    ero = phi_row(a, r0 + tid / CT, aux_w);
    e_j = j0 + tid % CT;
    ein = phi_epi_load<MODE>(a, ero, e_j);
    ebh = phi_bias_load(a, e_j);
  }

  // rows beyond the block are clamped to its last row (their sums are never used)
  const float* hrow[SK_RR];
#pragma unroll
  for (int i = 0; i < SK_RR; ++i) {
    const int r = r0 + min(rg * SK_RR + i, rows_here - 1);
    const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
    const int b = r - (int)pt * a.B;
    hrow[i] = a.u_in + (a.in.at(pt) * a.B + b) * H;
  }
  const WT* urow[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const int g = u / CT, j = min(j0 + u % CT, H - 1);
    urow[u] = (const WT*)a.U + ((long long)g * H + j) * H;
  }
  float acc[SK_RR][NU];
  skinny_dot<NU, WT>(acc, H, ks, ksl, urow, [&](int i, int k) { return ldg4(hrow[i] + k); });
  float v[VP];
#pragma unroll
  for (int q = 0; q < VP; ++q) v[q] = q < SK_RR * NU ? acc[q / NU][q % NU] : 0.f;
  skinny_reduce<VP>(v, red, rg, ks, ksl);
  __syncthreads();

  double nrm = 0.0;
  for (int e = tid; e < n_out; e += geo.nt) {
    const int row = e / CT, c = e % CT;
    const int j = j0 + c;
    if (j >= H) continue;
    const int grp = row / SK_RR, base = (row % SK_RR) * NU;
    const float sr = skinny_sum<VP>(red, grp, base + c, ksl);
    const float sz = skinny_sum<VP>(red, grp, base + CT + c, ksl);
    const float sn = skinny_sum<VP>(red, grp, base + 2 * CT + c, ksl);
    if (e == tid && epi) {
      phi_epi_finish<MODE>(a, ero, e_j, sr, sz, sn, ein, ebh, nrm,
                           (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
                               ? phi_row_coarse_kappa(a, r0 + row) : 0);
    } else {   // more outputs than threads (tiny K only)
      const PhiRow ro = phi_row(a, r0 + row, aux_w);
      phi_epi_finish<MODE>(a, ro, j, sr, sz, sn, phi_epi_load<MODE>(a, ro, j), phi_bias_load(a, j),
                           nrm,
                           (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
                               ? phi_row_coarse_kappa(a, r0 + row) : 0);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

// ---------------------------------------------------------------------------
// Few-row step on the matrix pipe
// ---------------------------------------------------------------------------
// The same step for up to 64 rows with the contraction on v_mfma_f32_16x16x4_f32, which sums
// over k inside the instruction: no partial sums travel between lanes, and a step needs a
// quarter of the waves of the vector form above (a dependent step waits for its slowest wave).
// A workgroup owns one block of 16 rows and FR_NC hidden columns; the three gates of those
// columns are the 16 columns of the MFMA block (3 x 5, one idle).  Its waves split K: wave w
// contracts k in [w kslice, (w + 1) kslice), every load of its slice issued before the first
// MFMA, and the 16 x 16 partial blocks meet in LDS.  Operand layout of the instruction: lane l
// supplies A[i = l % 16][k = l / 16] and B[k = l / 16][j = l % 16]; a lane loads four
// consecutive k of its row (k = 16 s + 4 (l / 16) + e, e = 0..3) and feeds four MFMAs, so A and
// B agree on the k each of them contracts; result register v of lane l is D[4 (l / 16) + v][l % 16].
constexpr int FR_NC = 5;       // hidden columns per workgroup
constexpr int FR_KB = 8;       // blocks of sixteen k whose loads a wave keeps in flight
constexpr int FR_MAXW = 8;     // waves per workgroup at most

template <int MODE, class WT>
__global__ __launch_bounds__(64 * FR_MAXW) void phi_fewrow_kernel(PhiArgs a, int kslice) {
  __shared__ float part[FR_MAXW][16][17];
  const int H = a.H;
  const int R = a.nk * a.B;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int nt = blockDim.x, nw = nt >> 6;
  const int li = lane & 15, kq = lane >> 4;
  const int j0 = blockIdx.x * FR_NC;
  const int r0 = blockIdx.y * 16;
  const int rows_here = min(16, R - r0);
  const int aux_w =
      (MODE == STEP_KAPPA || MODE == STEP_RELAX_KAPPA || MODE == STEP_RELAX_KAPPA2) ? a.kappa_width
                                                                                    : H;
  // this thread's output element (if any): its operands are requested first so that their
  // latency overlaps the contraction
  const int n_out = rows_here * FR_NC;
  const bool epi = tid < n_out && j0 + tid % FR_NC < H;
  int e_j = 0;
  PhiRow ero = {};
  PhiEpiIn ein = {};
  PhiBias ebh = {};
  if (epi) {
    ero = phi_row(a, r0 + tid / FR_NC, aux_w);
    e_j = j0 + tid % FR_NC;
    ein = phi_epi_load<MODE>(a, ero, e_j);
    ebh = phi_bias_load(a, e_j);
  }

  // A: state row of this lane (rows beyond the block are clamped; their sums are never used)
  const int r = r0 + min(li, rows_here - 1);
  const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
  const int b = r - (int)pt * a.B;
  const float* hrow = a.u_in + (a.in.at(pt) * a.B + b) * H;
  // B: weight row of this lane's MFMA column: gate li / FR_NC, hidden column j0 + li % FR_NC
  // (column 15 idles on a copy of column 14)
  const int lc = min(li, 3 * FR_NC - 1);
  const WT* urow = (const WT*)a.U +
                   ((long long)(lc / FR_NC) * H + min(j0 + lc % FR_NC, H - 1)) * H;

  // two accumulators: consecutive MFMAs do not wait for each other's result
  floatx4 acc = zero4(), acc1 = zero4();
  const int k_end = min(H, (wv + 1) * kslice);
  for (int kb = wv * kslice; kb < k_end; kb += 16 * FR_KB) {
    floatx4 av[FR_KB], bv[FR_KB];
#pragma unroll
    for (int s = 0; s < FR_KB; ++s) {
      const int k = kb + 16 * s + 4 * kq;
      const int kc = min(k, H - 4);                  // H is a multiple of 4
      av[s] = ldg4(hrow + kc);
      bv[s] = ldg4w(urow + kc);
    }
    // all loads of the slice are in flight before anything waits for one of them
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < FR_KB; ++s) {
      if (kb + 16 * s + 4 * kq >= k_end) av[s] = zero4();
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s][e], bv[s][e], acc, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s][e + 1], bv[s][e + 1], acc1, 0, 0, 0);
      }
    }
  }
  acc += acc1;
#pragma unroll
  for (int v = 0; v < 4; ++v) part[wv][4 * kq + v][li] = acc[v];
  __syncthreads();

  double nrm = 0.0;
  for (int e = tid; e < n_out; e += nt) {
    const int row = e / FR_NC, c = e % FR_NC;
    const int j = j0 + c;
    if (j >= H) continue;
    float sr = 0.f, sz = 0.f, sn = 0.f;
    for (int w = 0; w < nw; ++w) {
      sr += part[w][row][c];
      sz += part[w][row][FR_NC + c];
      sn += part[w][row][2 * FR_NC + c];
    }
    if (e == tid && epi) {
      phi_epi_finish<MODE>(a, ero, e_j, sr, sz, sn, ein, ebh, nrm,
                           (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
                               ? phi_row_coarse_kappa(a, r0 + row) : 0);
    } else {   // more outputs than threads (one-wave workgroups only)
      const PhiRow ro = phi_row(a, r0 + row, aux_w);
      phi_epi_finish<MODE>(a, ro, j, sr, sz, sn, phi_epi_load<MODE>(a, ro, j), phi_bias_load(a, j),
                           nrm,
                           (MODE == STEP_RELAX_KAPPA2 || MODE == STEP_RELAX_CK)
                               ? phi_row_coarse_kappa(a, r0 + row) : 0);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

typedef TileCfg<2, 2, 2, 1, 3> PhiBig;    // 128 rows x 64 hidden columns (x3 gates), 256 threads
typedef TileCfg<2, 2, 1, 1, 3> PhiMid;    //  64 rows x 64 hidden columns, 256 threads
// few rows:  32 rows x 32 hidden columns, 4 waves splitting K (slices of 128)
typedef TileCfg<1, 1, 1, 1, 3, 128, 1, 4> PhiSmall;
typedef TileCfgB<2, 2, 2, 1, 3, true> PhiBigB;
typedef TileCfgB<2, 2, 1, 1, 3, true> PhiMidB;
typedef TileCfgB<1, 1, 1, 1, 3, true, 4> PhiSmallB;
// the same tiles with the state as one bf16 term
typedef TileCfgB<2, 2, 2, 1, 3, true, 1, 1, 2, 1, 64, false> PhiBigF;
typedef TileCfgB<2, 2, 1, 1, 3, true, 1, 1, 2, 1, 64, false> PhiMidF;
typedef TileCfgB<1, 1, 1, 1, 3, true, 4, 1, 2, 1, 64, false> PhiSmallF;
// 64 x 64 with two groups of four waves splitting K (slices of 128): half the dependent slices
// per workgroup, for launches whose tiles do not fill the CUs twice anyway (one workgroup per
// CU: 110 KB of LDS with both groups' sums staged); 22.5 -> 20.3 us at 512 rows x 1024
typedef TileCfgB<2, 2, 1, 1, 3, true, 2, 1, 1, 1, 64, false> PhiMidFK;
// three-term operands: K-slices of 32 keep two workgroups' tiles in a CU's LDS
typedef TileCfgB<2, 2, 2, 1, 3, true, 1, 1, 2, 3, 32> PhiBigS;
typedef TileCfgB<2, 2, 1, 1, 3, true, 1, 1, 2, 3, 32> PhiMidS;
typedef TileCfgB<1, 1, 1, 1, 3, true, 4, 1, 2, 3, 32> PhiSmallS;

#define MG_LAUNCH_BY_MODE(KERNEL, ...)                                                   \
  switch (a.mode) {                                                                      \
    case STEP_RELAX:                                                                     \
      if (a.zero_from > 0)                                                               \
        hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX, true>), grid, block, 0, s, a); \
      else                                                                               \
        hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX>), grid, block, 0, s, a);     \
      break;                                                                             \
    case STEP_RESID:                                                                     \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RESID>), grid, block, 0, s, a);       \
      break;                                                                             \
    case STEP_RHS:                                                                       \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RHS>), grid, block, 0, s, a);         \
      break;                                                                             \
    case STEP_RELAX_KAPPA:                                                               \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX_KAPPA>), grid, block, 0, s, a); \
      break;                                                                             \
    case STEP_RELAX_CK:                                                                  \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX_CK>), grid, block, 0, s, a);    \
      break;                                                                             \
    case STEP_RELAX_KAPPA2:                                                              \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX_KAPPA2>), grid, block, 0, s, a); \
      break;                                                                             \
    case STEP_RELAX_RHS:                                                                 \
      if (a.zero_from > 0)                                                               \
        hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX_RHS, true>), grid, block, 0, s, a); \
      else                                                                               \
        hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_RELAX_RHS>), grid, block, 0, s, a); \
      break;                                                                             \
    default:                                                                             \
      hipLaunchKernelGGL((KERNEL<__VA_ARGS__, STEP_KAPPA>), grid, block, 0, s, a);       \
  }

template <class C, class CB, class CS, class CF>
static void launch_phi_cfg(const PhiArgs& a, hipStream_t s) {
  const long long R = (long long)a.nk * a.B;
  static_assert(CF::TM == CB::TM && CF::TN == CB::TN, "tile shapes must agree");
  if (a.bf16 == 2) {
    dim3 grid((unsigned)xcd_grid((R + CS::TM - 1) / CS::TM, (a.H + CS::TN - 1) / CS::TN));
    dim3 block(CS::NT);
    MG_LAUNCH_BY_MODE(phi_step_kernel_bf16, CS)
  } else if (a.bf16 && a.one_term) {
    dim3 grid((unsigned)xcd_grid((R + CF::TM - 1) / CF::TM, (a.H + CF::TN - 1) / CF::TN));
    dim3 block(CF::NT);
    MG_LAUNCH_BY_MODE(phi_step_kernel_bf16, CF)
  } else if (a.bf16) {
    dim3 grid((unsigned)xcd_grid((R + CB::TM - 1) / CB::TM, (a.H + CB::TN - 1) / CB::TN));
    dim3 block(CB::NT);
    MG_LAUNCH_BY_MODE(phi_step_kernel_bf16, CB)
  } else {
    dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (a.H + C::TN - 1) / C::TN));
    dim3 block(C::NT);
    MG_LAUNCH_BY_MODE(phi_step_kernel, C)
  }
}

constexpr int PHI_SK_ROWS = 32;   // rows per workgroup of the few-row forward step

static int phi_sk_rows(long long R) { return R < PHI_SK_ROWS ? (int)R : PHI_SK_ROWS; }

template <int CT, int MODE>
static void launch_phi_skinny_mode(const PhiArgs& a, dim3 grid, hipStream_t s) {
  const int rb = phi_sk_rows((long long)a.nk * a.B);
  const dim3 block(sk_geom(rb, a.H).nt);
  if (a.bf16 == 1)
    hipLaunchKernelGGL((phi_skinny_kernel<CT, MODE, bf16_t>), grid, block, 0, s, a, rb);
  else
    hipLaunchKernelGGL((phi_skinny_kernel<CT, MODE, float>), grid, block, 0, s, a, rb);
}

template <int MODE>
static void launch_phi_fewrow_mode(const PhiArgs& a, hipStream_t s) {
  const int R = a.nk * a.B;
  // waves per workgroup: K slices of 128 (two blocks of loads in flight at most beyond that)
  int nw = (a.H + 127) / 128;
  nw = nw < 1 ? 1 : (nw > FR_MAXW ? FR_MAXW : nw);
  const int kslice = ((a.H + nw - 1) / nw + 15) / 16 * 16;
  const dim3 grid((unsigned)((a.H + FR_NC - 1) / FR_NC), (unsigned)((R + 15) / 16));
  const dim3 block(64 * nw);
  if (a.bf16 == 1)
    hipLaunchKernelGGL((phi_fewrow_kernel<MODE, bf16_t>), grid, block, 0, s, a, kslice);
  else
    hipLaunchKernelGGL((phi_fewrow_kernel<MODE, float>), grid, block, 0, s, a, kslice);
}

static void launch_phi_fewrow(const PhiArgs& a, hipStream_t s) {
  switch (a.mode) {
    case STEP_RELAX: launch_phi_fewrow_mode<STEP_RELAX>(a, s); break;
    case STEP_RESID: launch_phi_fewrow_mode<STEP_RESID>(a, s); break;
    case STEP_RHS: launch_phi_fewrow_mode<STEP_RHS>(a, s); break;
    case STEP_RELAX_KAPPA: launch_phi_fewrow_mode<STEP_RELAX_KAPPA>(a, s); break;
    case STEP_RELAX_RHS: launch_phi_fewrow_mode<STEP_RELAX_RHS>(a, s); break;
    case STEP_RELAX_KAPPA2: launch_phi_fewrow_mode<STEP_RELAX_KAPPA2>(a, s); break;
    case STEP_RELAX_CK: launch_phi_fewrow_mode<STEP_RELAX_CK>(a, s); break;
    default: launch_phi_fewrow_mode<STEP_KAPPA>(a, s);
  }
}

template <int CT>
static void launch_phi_skinny(const PhiArgs& a, dim3 grid, hipStream_t s) {
  switch (a.mode) {
    case STEP_RELAX: launch_phi_skinny_mode<CT, STEP_RELAX>(a, grid, s); break;
    case STEP_RESID: launch_phi_skinny_mode<CT, STEP_RESID>(a, grid, s); break;
    case STEP_RHS: launch_phi_skinny_mode<CT, STEP_RHS>(a, grid, s); break;
    case STEP_RELAX_KAPPA: launch_phi_skinny_mode<CT, STEP_RELAX_KAPPA>(a, grid, s); break;
    case STEP_RELAX_RHS: launch_phi_skinny_mode<CT, STEP_RELAX_RHS>(a, grid, s); break;
    case STEP_RELAX_KAPPA2: launch_phi_skinny_mode<CT, STEP_RELAX_KAPPA2>(a, grid, s); break;
    case STEP_RELAX_CK: launch_phi_skinny_mode<CT, STEP_RELAX_CK>(a, grid, s); break;
    default: launch_phi_skinny_mode<CT, STEP_KAPPA>(a, grid, s);
  }
}

// MGRIT_FEWROW_VECTOR=1 in the environment selects the vector-FMA form of the few-row step
// (kept for widths below 16 and for comparison)
static bool getenv_vector_fewrow() {
  static const bool v = [] {
    const char* e = std::getenv("MGRIT_FEWROW_VECTOR");
    return e && e[0] == '1';
  }();
  return v;
}

hipError_t launch_phi_step(const PhiArgs& a, hipStream_t s) {
  if (a.nk <= 0) return hipSuccess;
  if (a.propagator == PROP_ODE_DEMO) return launch_ode_step(a, s);
  if (prop_is_lstm(a.propagator)) return launch_lstm_step(a, s);
  const long long R = (long long)a.nk * a.B;
  auto tiles = [&](int tm, int tn) { return ((R + tm - 1) / tm) * ((a.H + tn - 1) / tn); };
  const int kind = R <= 2 * SK_MAXROWS ? 4 : 0;
  // a launch that skips the contraction of its zero-input tiles is its own shape class for
  // the event timings (mode + 16), and only the rows it contracts count as work
  prof_begin(kind, s, R, kind == 0 && a.zero_from > 0 ? a.mode + 16 : a.mode);
  long long rows_done = R;
  auto contracted = [&](int tm) {
    if (a.zero_from > 0) rows_done = std::min<long long>(R, (a.zero_from + tm - 1) / tm * tm);
  };
  if (R <= 2 * SK_MAXROWS && a.H >= 16 && !getenv_vector_fewrow()) {
    launch_phi_fewrow(a, s);
  } else if (R <= 2 * SK_MAXROWS) {
    // two hidden columns (six weight rows) per workgroup measured best from H = 512 up
    // (6.2 us per step at 32 rows x 512, 5.5 at 4 rows x 1024; four columns: +0.5 us)
    const int rb = phi_sk_rows(R);
    const int nrb = (int)((R + rb - 1) / rb);
    const int ct = a.H * nrb >= 512 ? 2 : 1;
    dim3 grid((unsigned)((a.H + ct - 1) / ct), (unsigned)nrb);
    if (ct == 2)
      launch_phi_skinny<2>(a, grid, s);
    else
      launch_phi_skinny<1>(a, grid, s);
  } else if (tiles(PhiBig::TM, PhiBig::TN) >= 384) {
    contracted(PhiBig::TM);
    launch_phi_cfg<PhiBig, PhiBigB, PhiBigS, PhiBigF>(a, s);
  } else if (R > 32 && tiles(PhiMid::TM, PhiMid::TN) >= 128) {
    contracted(PhiMid::TM);
    if (a.bf16 == 1 && a.one_term && tiles(PhiMid::TM, PhiMid::TN) <= 256)
      launch_phi_cfg<PhiMid, PhiMidB, PhiMidS, PhiMidFK>(a, s);
    else
      launch_phi_cfg<PhiMid, PhiMidB, PhiMidS, PhiMidF>(a, s);
  } else {
    contracted(PhiSmall::TM);
    launch_phi_cfg<PhiSmall, PhiSmallB, PhiSmallS, PhiSmallF>(a, s);
  }
  prof_end(kind, 6.0 * (double)rows_done * a.H * a.H, 20.0 * (double)R * a.H, s);
  return hipGetLastError();
}

}  // namespace mg
