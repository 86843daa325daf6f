// Forward-Euler level step of the demonstration ODE of the paper's appendix
// ("Why does MGRIT work?", Eq. 17),
//   dh/dt = -h/2 + sigmoid(A h + B d(t) + b),
//   Phi_dt(h; d) = h + dt * (-h/2 + sigmoid(A h + P)),   P = B d + b  (precomputed),
// as a second propagator behind the forward MGRIT drivers: the same launch
// description (PhiArgs: U = A[H,H], P rows of width H, gamma = dt of the level, b_h
// unused) and the same epilogue modes as the GRU step, forward propagation only.
#include "common.h"
#include "gates.h"
#include "gemm_core.h"
#include "skinny.h"

namespace mg {

// Element offsets (column 0) of one row (level point, batch element) of a launch:
// input state, projection row, out/cur/g, coarse array.
struct OdeRow {
  long long in, p, o, a;
};
__device__ inline OdeRow ode_row(const PhiArgs& a, long long r) {
  const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
  const int b = (int)(r - pt * a.B);
  OdeRow ro;
  ro.in = (a.in.at(pt) * a.B + b) * a.H;
  ro.p = (a.p.at(pt) * a.B + b) * a.H;
  ro.o = (a.o.at(pt) * a.B + b) * a.H;
  ro.a = (a.a.at(pt) * a.B + b) * a.H;
  // (row offsets are multiples of four elements: bit 0 marks the coarse points of ff_cf / ff_rem)
  if (a.ff_cf > 0 && a.a.at(pt) % a.ff_cf == a.ff_rem) ro.a |= 1;
  return ro;
}

struct OdeEpiIn4 {
  floatx4 p, h, gval, cur;
};
struct OdeEpiExtra4 {     // STEP_RELAX_RHS (p2, cur2) and STEP_RESID with resid_adds (prep)
  floatx4 p2, cur2, prep;
};

// Epilogue of one MFMA tile over the staged sums (A h): the Euler update and the
// mode's outputs, moved as float4 (see EpiStage).
template <class C, int MODE>
__device__ inline void ode_tile_epilogue(const PhiArgs& a, Acc<C>& acc, const OdeRow* rowtab,
                                         float* stage, long long m0, int n0, long long R,
                                         double& nrm) {
  typedef EpiStage<C> E;
  const int H = a.H;
  const int c4 = E::col4();
  const int j = n0 + c4 * 4;
  const bool colok = E::active() && j < H;
  const int jc = colok ? j : H - 4;                     // clamped columns are never stored
  const float dt = a.gamma;
#pragma unroll
  for (int ba = 0; ba < C::BM; ++ba) {
    __syncthreads();                                    // staging area no longer read
    E::write(acc, ba, stage);
    OdeEpiIn4 in[E::ITEMS];
    constexpr bool EXTRA = MODE == STEP_RELAX_RHS || MODE == STEP_RESID;
    OdeEpiExtra4 ex[EXTRA ? E::ITEMS : 1];
    long long oo[E::ITEMS], oa[E::ITEMS];
    int trow[E::ITEMS];
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      trow[it] = E::tile_row(E::staged_row(it), ba);
      const OdeRow ro = rowtab[trow[it]];               // rows beyond the launch hold its last row
      oo[it] = ro.o;
      oa[it] = ro.a;
      in[it].p = ldg4(a.P + ro.p + jc);
      in[it].h = ldg4(a.u_in + ro.in + jc);
      in[it].gval = a.g ? ldg4(a.g + ro.o + jc) : zero4();
      in[it].cur = (MODE == STEP_RESID || MODE == STEP_RHS) ? ldg4(a.u + ro.o + jc) : zero4();
      if (MODE == STEP_RELAX_RHS) {
        ex[it].p2 = ldg4(a.P + ro.p + a.dp2 + jc);
        ex[it].cur2 = ldg4(a.u + ro.o + a.do2 + jc);
      }
      if (MODE == STEP_RESID)
        ex[it].prep = a.resid_adds ? ldg4(a.gc + (ro.a & ~1LL) + jc) : zero4();
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      const floatx4 dot = E::read(stage, 0, E::staged_row(it), c4);
      if (!colok || m0 + trow[it] >= R) continue;
      floatx4 hn;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float h = in[it].h[i];
        hn[i] = h + dt * (sigmoidf_(dot[i] + in[it].p[i]) - 0.5f * h);
      }
      const long long oi = oo[it] + j;
      if (MODE == STEP_RELAX) {
        *reinterpret_cast<floatx4*>(a.u + oi) = hn + in[it].gval;
      } else if (MODE == STEP_RELAX_RHS) {
        *reinterpret_cast<floatx4*>(a.u + oi) = hn + in[it].gval;
        // the coarse level's step from the same state: same sums, its own data and step size
        floatx4 hn2;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float h = in[it].h[i];
          hn2[i] = h + a.gamma2 * (sigmoidf_(dot[i] + ex[it].p2[i]) - 0.5f * h);
        }
        *reinterpret_cast<floatx4*>(a.gc + oa[it] + j) = ex[it].cur2 - hn2;
      } else if (MODE == STEP_RESID) {
        const floatx4 res = in[it].cur - hn - in[it].gval;
        const long long ai = (oa[it] & ~1LL) + j;
        *reinterpret_cast<floatx4*>(a.gc + ai) = ex[it].prep + (-res);
        // cur - r at the marked points
        *reinterpret_cast<floatx4*>(a.uc + ai) = (oa[it] & 1) ? in[it].cur - res : in[it].cur;
#pragma unroll
        for (int i = 0; i < 4; ++i) nrm += (double)res[i] * (double)res[i];
      } else {  // STEP_RHS
        *reinterpret_cast<floatx4*>(a.g + oi) = (in[it].cur - hn) + in[it].gval;
      }
    }
  }
}

// out[R,H] rows = (level point, batch element); the contraction is h[R,H] . A[H,H]^T on
// the fp32 MFMA tile core, one workgroup per (row tile, column tile).
template <class C, int MODE>
__global__ __launch_bounds__(C::NT, C::MINWG) void ode_step_kernel(PhiArgs a) {
  constexpr int LDSF =
      C::LDS_FLOATS > EpiStage<C>::FLOATS ? C::LDS_FLOATS : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float lds[LDSF];
  const int H = a.H, B = a.B;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  __shared__ OdeRow rowtab[C::TM];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = ode_row(a, r);
  }
  // (visible to all waves after the barriers inside the contraction)

  const float* arow[C::A_CHUNKS];
  const float* brow[C::B_CHUNKS];
#pragma unroll
  for (int s = 0; s < C::A_CHUNKS; ++s) {
    long long r = m0 + chunk_row<C>(s);
    if (r >= R) r = R - 1;     // clamped rows are never stored
    const long long pt = (unsigned)r / (unsigned)B;
    const int b = (int)(r - pt * B);
    arow[s] = a.u_in + (a.in.at(pt) * B + b) * H;
  }
#pragma unroll
  for (int s = 0; s < C::B_CHUNKS; ++s) {
    int j = n0 + chunk_row<C>(s);
    if (j >= H) j = H - 1;
    brow[s] = (const float*)a.U + (long long)j * H;
  }
  Acc<C> acc;
  acc.zero();
  auto la = [&](int s, int k) { return ldg4(arow[s] + k); };
  auto lb = [&](int s, int k) { return ldg4(brow[s] + k); };
  if (H % C::TK == 0)
    gemm_nt_tile<C, false>(acc, H, la, lb, Identity4(), Identity4(), lds);
  else
    gemm_nt_tile<C, true>(acc, H, la, lb, Identity4(), Identity4(), lds);

  double nrm = 0.0;
  ode_tile_epilogue<C, MODE>(a, acc, rowtab, lds, m0, n0, R, nrm);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// Few rows (the coarsest level's serial propagation, a serial scan over a small batch):
// the vector-FMA form of skinny.h.  A workgroup owns a block of rows x CT columns of A h;
// its threads split K, the partial sums meet through the lane butterfly and LDS, and
// thread (row, column) applies the update.  Epilogue operands are requested before the
// dot products.
struct OdeEpiIn {
  float p, h, gval, cur;
  float p2, cur2, prep;     // STEP_RELAX_RHS / STEP_RESID with resid_adds (see OdeEpiExtra4)
};
template <int MODE>
__device__ inline OdeEpiIn ode_epi_load(const PhiArgs& a, const OdeRow& ro, int j) {
  OdeEpiIn e;
  e.p = a.P[ro.p + j];
  e.h = a.u_in[ro.in + j];
  e.gval = a.g ? a.g[ro.o + j] : 0.f;
  e.cur = (MODE == STEP_RESID || MODE == STEP_RHS) ? a.u[ro.o + j] : 0.f;
  e.p2 = e.cur2 = e.prep = 0.f;
  if (MODE == STEP_RELAX_RHS) {
    e.p2 = a.P[ro.p + a.dp2 + j];
    e.cur2 = a.u[ro.o + a.do2 + j];
  }
  if (MODE == STEP_RESID && a.resid_adds) e.prep = a.gc[(ro.a & ~1LL) + j];
  return e;
}
template <int MODE>
__device__ inline void ode_epi_finish(const PhiArgs& a, const OdeRow& ro, int j, float dot,
                                      const OdeEpiIn& e, double& nrm) {
  const float hn = e.h + a.gamma * (sigmoidf_(dot + e.p) - 0.5f * e.h);
  const long long oi = ro.o + j;
  if (MODE == STEP_RELAX) {
    a.u[oi] = hn + e.gval;
  } else if (MODE == STEP_RELAX_RHS) {
    a.u[oi] = hn + e.gval;
    const float hn2 = e.h + a.gamma2 * (sigmoidf_(dot + e.p2) - 0.5f * e.h);
    a.gc[ro.a + j] = e.cur2 - hn2;
  } else if (MODE == STEP_RESID) {
    const float res = e.cur - hn - e.gval;
    const long long ai = (ro.a & ~1LL) + j;
    a.gc[ai] = a.resid_adds ? e.prep + (-res) : -res;
    a.uc[ai] = (ro.a & 1) ? e.cur - res : e.cur;       // cur - r at the marked points
    nrm += (double)res * (double)res;
  } else {  // STEP_RHS
    a.g[oi] = (e.cur - hn) + e.gval;
  }
}

constexpr int ODE_SK_ROWS = 32;   // rows per workgroup of the few-row step

template <int CT, int MODE>
__global__ __launch_bounds__(SK_MAXNT) void ode_skinny_kernel(PhiArgs a, int rows_block) {
  constexpr int VP = sk_pow2_ceil(SK_RR * CT);
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

  const int n_out = rows_here * CT;
  const bool epi = tid < n_out && j0 + tid % CT < H;
  int e_j = 0;
  OdeRow ero = {};
  OdeEpiIn ein = {};
  if (epi) {
    ero = ode_row(a, r0 + tid / CT);
    e_j = j0 + tid % CT;
    ein = ode_epi_load<MODE>(a, ero, e_j);
  }

  // rows beyond the block are clamped to its last row (their sums are never used)
  const float* hrow[SK_RR];
#pragma unroll
  for (int i = 0; i < SK_RR; ++i) {
    const int r = r0 + min(rg * SK_RR + i, rows_here - 1);
    const long long pt = (unsigned)r / (unsigned)a.B;
    const int b = r - (int)pt * a.B;
    hrow[i] = a.u_in + (a.in.at(pt) * a.B + b) * H;
  }
  const float* wrow[CT];
#pragma unroll
  for (int u = 0; u < CT; ++u) wrow[u] = (const float*)a.U + (long long)min(j0 + u, H - 1) * H;
  float acc[SK_RR][CT];
  skinny_dot<CT, float>(acc, H, ks, ksl, wrow, [&](int i, int k) { return ldg4(hrow[i] + k); });
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
      ode_epi_finish<MODE>(a, ero, e_j, dot, ein, nrm);
    } else {   // more outputs than threads (tiny K only)
      const OdeRow ro = ode_row(a, r0 + row);
      ode_epi_finish<MODE>(a, ro, j, dot, ode_epi_load<MODE>(a, ro, j), nrm);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

// The few-row step on the matrix pipe (v_mfma_f32_16x16x4_f32), as the GRU's phi_fewrow_kernel: a
// workgroup owns 16 rows and OFR_NC columns of A h (the other MFMA columns idle on copies of
// the last one: the step is bound by latency, not by the pipe); its waves split K, each wave
// with all loads of its slice in flight before its first MFMA; the partial blocks meet in LDS
// and thread (row, column) applies the update.  Lane l supplies A[i = l % 16][k = l / 16] and
// B[k = l / 16][j = l % 16]; result register v of lane l is D[4 (l / 16) + v][l % 16].
constexpr int OFR_NC = 5;      // columns per workgroup (as many workgroups as the GRU's step has)
constexpr int OFR_KB = 8;      // blocks of sixteen k whose loads a wave keeps in flight
constexpr int OFR_MAXW = 8;    // waves per workgroup at most

template <int MODE>
__global__ __launch_bounds__(64 * OFR_MAXW) void ode_fewrow_kernel(PhiArgs a, int kslice) {
  __shared__ float part[OFR_MAXW][16][17];
  const int H = a.H;
  const int R = a.nk * a.B;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int nt = blockDim.x, nw = nt >> 6;
  const int li = lane & 15, kq = lane >> 4;
  const int j0 = blockIdx.x * OFR_NC;
  const int r0 = blockIdx.y * 16;
  const int rows_here = min(16, R - r0);

  // this thread's output element (if any): its operands are requested before the contraction
  const int n_out = rows_here * OFR_NC;
  const bool epi = tid < n_out && j0 + tid % OFR_NC < H;
  int e_j = 0;
  OdeRow ero = {};
  OdeEpiIn ein = {};
  if (epi) {
    ero = ode_row(a, r0 + tid / OFR_NC);
    e_j = j0 + tid % OFR_NC;
    ein = ode_epi_load<MODE>(a, ero, e_j);
  }

  const int r = r0 + min(li, rows_here - 1);         // rows beyond the block are clamped
  const long long pt = (unsigned)r / (unsigned)a.B;
  const int b = r - (int)pt * a.B;
  const float* hrow = a.u_in + (a.in.at(pt) * a.B + b) * H;
  const float* urow = (const float*)a.U + (long long)min(j0 + min(li, OFR_NC - 1), H - 1) * H;

  floatx4 acc = zero4(), acc1 = zero4();
  const int k_end = min(H, (wv + 1) * kslice);
  for (int kb = wv * kslice; kb < k_end; kb += 16 * OFR_KB) {
    floatx4 av[OFR_KB], bv[OFR_KB];
#pragma unroll
    for (int s = 0; s < OFR_KB; ++s) {
      const int k = kb + 16 * s + 4 * kq;
      const int kc = min(k, H - 4);                  // H is a multiple of 4
      av[s] = ldg4(hrow + kc);
      bv[s] = ldg4(urow + kc);
    }
    __builtin_amdgcn_sched_barrier(0);               // all loads in flight before the first wait
#pragma unroll
    for (int s = 0; s < OFR_KB; ++s) {
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
    const int row = e / OFR_NC, c = e % OFR_NC;
    const int j = j0 + c;
    if (j >= H) continue;
    float dot = 0.f;
    for (int w = 0; w < nw; ++w) dot += part[w][row][c];
    if (e == tid && epi) {
      ode_epi_finish<MODE>(a, ero, e_j, dot, ein, nrm);
    } else {   // more outputs than threads (one-wave workgroups only)
      const OdeRow ro = ode_row(a, r0 + row);
      ode_epi_finish<MODE>(a, ro, j, dot, ode_epi_load<MODE>(a, ro, j), nrm);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

static void launch_ode_fewrow(const PhiArgs& a, hipStream_t s) {
  const int R = a.nk * a.B, H = a.H;
  int nw = (H + 127) / 128;
  nw = nw < 1 ? 1 : (nw > OFR_MAXW ? OFR_MAXW : nw);
  const int kslice = ((H + nw - 1) / nw + 15) / 16 * 16;
  const dim3 grid((unsigned)((H + OFR_NC - 1) / OFR_NC), (unsigned)((R + 15) / 16));
  const dim3 block(64 * nw);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL(ode_fewrow_kernel<STEP_RELAX>, grid, block, 0, s, a, kslice);
  else if (a.mode == STEP_RELAX_RHS)
    hipLaunchKernelGGL(ode_fewrow_kernel<STEP_RELAX_RHS>, grid, block, 0, s, a, kslice);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL(ode_fewrow_kernel<STEP_RESID>, grid, block, 0, s, a, kslice);
  else
    hipLaunchKernelGGL(ode_fewrow_kernel<STEP_RHS>, grid, block, 0, s, a, kslice);
}

template <int CT>
static void launch_ode_skinny(const PhiArgs& a, dim3 grid, int rb, hipStream_t s) {
  const dim3 block(sk_geom(rb, a.H).nt);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL((ode_skinny_kernel<CT, STEP_RELAX>), grid, block, 0, s, a, rb);
  else if (a.mode == STEP_RELAX_RHS)
    hipLaunchKernelGGL((ode_skinny_kernel<CT, STEP_RELAX_RHS>), grid, block, 0, s, a, rb);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL((ode_skinny_kernel<CT, STEP_RESID>), grid, block, 0, s, a, rb);
  else
    hipLaunchKernelGGL((ode_skinny_kernel<CT, STEP_RHS>), grid, block, 0, s, a, rb);
}

typedef TileCfg<2, 2, 2, 2, 1> OdeBig;                  // 128 x 128, 256 threads
typedef TileCfg<2, 2, 1, 1, 1> OdeMid;                  //  64 x 64, 256 threads
typedef TileCfg<1, 1, 1, 1, 1, 128, 1, 4> OdeSmall;     //  32 x 32, 4 waves splitting K

template <class C>
static void launch_ode_cfg(const PhiArgs& a, hipStream_t s) {
  const long long R = (long long)a.nk * a.B;
  dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (a.H + C::TN - 1) / C::TN));
  dim3 block(C::NT);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL((ode_step_kernel<C, STEP_RELAX>), grid, block, 0, s, a);
  else if (a.mode == STEP_RELAX_RHS)
    hipLaunchKernelGGL((ode_step_kernel<C, STEP_RELAX_RHS>), grid, block, 0, s, a);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL((ode_step_kernel<C, STEP_RESID>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((ode_step_kernel<C, STEP_RHS>), grid, block, 0, s, a);
}

// Up to 64 rows: the few-row kernel.  Above: tile shape by the number of workgroups it
// gives, 128 x 128 tiles when they alone fill the chip, 64 x 64 below that, else 32 x 32
// tiles whose four waves split K.
hipError_t launch_ode_step(const PhiArgs& a, hipStream_t s) {
  if (a.nk <= 0) return hipSuccess;
  if (a.mode != STEP_RELAX && a.mode != STEP_RESID && a.mode != STEP_RHS &&
      a.mode != STEP_RELAX_RHS)
    return hipErrorInvalidValue;
  const long long R = (long long)a.nk * a.B;
  auto tiles = [&](int tm, int tn) { return ((R + tm - 1) / tm) * ((a.H + tn - 1) / tn); };
  prof_begin(8, s, R, a.mode);
  if (R <= 2 * SK_MAXROWS && R >= 16 && a.H >= 16) {
    // (with fewer rows than one MFMA block the vector form below issues a quarter of the loads
    // and measured faster: 4.3 against 4.6 us per step at 4 rows x 1024)
    launch_ode_fewrow(a, s);
  } else if (R <= 2 * SK_MAXROWS) {
    // as many workgroups as the GRU's few-row step has at the same width: H / 2 there
    // (two columns of three gates), H / 4 or H / 2 here
    const int rb = R < ODE_SK_ROWS ? (int)R : ODE_SK_ROWS;
    const int nrb = (int)((R + rb - 1) / rb);
    const int ct = a.H * nrb >= 1024 ? 4 : (a.H * nrb >= 256 ? 2 : 1);
    dim3 grid((unsigned)((a.H + ct - 1) / ct), (unsigned)nrb);
    if (ct == 4)
      launch_ode_skinny<4>(a, grid, rb, s);
    else if (ct == 2)
      launch_ode_skinny<2>(a, grid, rb, s);
    else
      launch_ode_skinny<1>(a, grid, rb, s);
  } else if (tiles(OdeBig::TM, OdeBig::TN) >= 384)
    launch_ode_cfg<OdeBig>(a, s);
  else if (R > 32 && tiles(OdeMid::TM, OdeMid::TN) >= 256)
    launch_ode_cfg<OdeMid>(a, s);
  else
    launch_ode_cfg<OdeSmall>(a, s);
  prof_end(8, 2.0 * (double)R * a.H * a.H, 16.0 * (double)R * a.H, s);
  return hipGetLastError();
}

}  // namespace mg
