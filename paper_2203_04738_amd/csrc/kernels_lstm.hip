// Level step of an LSTM layer as a third propagator behind the forward MGRIT drivers (the
// extension the paper's conclusion names; it gives no equations).  The step is derived the way
// Sec. 3.3 derives the Implicit GRU: the cell is read as a forward-Euler step of
//   dc/dt = -(1 - f) c + i g,   dh/dt = -h + o tanh(c),
// gates i, f, o = sigmoid(.), g = tanh(.) of P + U h + b_h at (x_t, h_{t-1}), and the decay terms
// are taken implicitly:
//   implicit:  c' = (c + gamma i g) / (1 + gamma (1 - f)),   h' = (h + gamma o tanh(c')) / (1 + gamma)
//   explicit:  c' = c + gamma (-(1 - f) c + i g),            h' = h + gamma (-h + o tanh(c'))
// (the explicit step with gamma = 1 is the standard LSTM cell).  The state of the time
// integration is the pair (h, c): state rows are 2H wide, h in columns 0..H-1, c in H..2H-1.
// Launch description: PhiArgs with H = state width 2H_hidden, U = U[4H_h, H_h] (gate order
// i, f, g, o), P rows of width 4H_h, gamma = step size of the level.  Epilogue modes STEP_RELAX,
// STEP_RESID, STEP_RHS; forward propagation only.
#include "common.h"
#include "gates.h"
#include "gemm_core.h"
#include "skinny.h"

namespace mg {

// Element offsets (column 0) of one row (level point, batch element) of a launch: input state
// row, projection row, out/cur/g row, coarse row.
struct LstmRow {
  long long in, p, o, a;
};
__device__ inline LstmRow lstm_row(const PhiArgs& a, long long r) {
  const long long pt = (unsigned)r / (unsigned)a.B;   // rows < 2^31: 32-bit division
  const int b = (int)(r - pt * a.B);
  LstmRow ro;
  ro.in = (a.in.at(pt) * a.B + b) * a.H;
  ro.p = (a.p.at(pt) * a.B + b) * (2LL * a.H);        // 4 H_hidden
  ro.o = (a.o.at(pt) * a.B + b) * a.H;
  ro.a = (a.a.at(pt) * a.B + b) * a.H;
  return ro;
}

// New (h, c) of one element from the four recurrent sums.
struct LstmNew {
  float h, c;
};
__device__ inline LstmNew lstm_elem(float gamma, bool implicit, float si, float sf, float sg,
                                    float so, float h, float c) {
  const float ig = sigmoidf_(si);
  const float fg = sigmoidf_(sf);
  const float gg = tanhf_(sg);
  const float og = sigmoidf_(so);
  LstmNew n;
  if (implicit) {
    n.c = (c + gamma * ig * gg) * fast_rcp(1.0f + gamma * (1.0f - fg));
    n.h = (h + gamma * og * tanhf_(n.c)) * fast_rcp(1.0f + gamma);
  } else {
    n.c = c + gamma * (ig * gg - (1.0f - fg) * c);
    n.h = h + gamma * (og * tanhf_(n.c) - h);
  }
  return n;
}

struct LstmEpiIn4 {
  floatx4 p[4], h, c, gh, gc, curh, curc;
};

// Epilogue of one MFMA tile over the staged sums (see EpiStage): gates, update and the mode's
// outputs for both halves of the state, moved as float4.
template <class C, int MODE>
__device__ inline void lstm_tile_epilogue(const PhiArgs& a, Acc<C>& acc, const LstmRow* rowtab,
                                          float* stage, long long m0, int n0, long long R,
                                          double& nrm) {
  typedef EpiStage<C> E;
  const int H = a.H / 2;
  const int c4 = E::col4();
  const int j = n0 + c4 * 4;
  const bool colok = E::active() && j < H;
  const int jc = colok ? j : H - 4;                     // clamped columns are never stored
  floatx4 bias[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) bias[g] = ldg4(a.b_h + g * H + jc);
  const float gamma = a.gamma;
  const bool implicit = a.propagator == PROP_LSTM_IMPLICIT;
#pragma unroll
  for (int ba = 0; ba < C::BM; ++ba) {
    __syncthreads();                                    // staging area no longer read
    E::write(acc, ba, stage);
    LstmEpiIn4 in[E::ITEMS];
    long long oo[E::ITEMS], oa[E::ITEMS];
    int trow[E::ITEMS];
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      trow[it] = E::tile_row(E::staged_row(it), ba);
      const LstmRow ro = rowtab[trow[it]];              // rows beyond the launch hold its last row
      oo[it] = ro.o;
      oa[it] = ro.a;
      const float* pp = a.P + ro.p + jc;
#pragma unroll
      for (int g = 0; g < 4; ++g) in[it].p[g] = ldg4_stream(pp + g * H);
      in[it].h = ldg4(a.u_in + ro.in + jc);
      in[it].c = ldg4(a.u_in + ro.in + H + jc);
      in[it].gh = a.g ? ldg4(a.g + ro.o + jc) : zero4();
      in[it].gc = a.g ? ldg4(a.g + ro.o + H + jc) : zero4();
      if (MODE == STEP_RESID || MODE == STEP_RHS) {
        in[it].curh = ldg4(a.u + ro.o + jc);
        in[it].curc = ldg4(a.u + ro.o + H + jc);
      } else {
        in[it].curh = in[it].curc = zero4();
      }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < E::ITEMS; ++it) {
      const int rp = E::staged_row(it);
      floatx4 s[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) s[g] = E::read(stage, g, rp, c4) + in[it].p[g] + bias[g];
      if (!colok || m0 + trow[it] >= R) continue;
      floatx4 hn, cn;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const LstmNew n = lstm_elem(gamma, implicit, s[0][i], s[1][i], s[2][i], s[3][i],
                                    in[it].h[i], in[it].c[i]);
        hn[i] = n.h;
        cn[i] = n.c;
      }
      const long long oi = oo[it] + j;
      if (MODE == STEP_RELAX) {
        *reinterpret_cast<floatx4*>(a.u + oi) = hn + in[it].gh;
        *reinterpret_cast<floatx4*>(a.u + oi + H) = cn + in[it].gc;
      } else if (MODE == STEP_RESID) {
        const floatx4 rh = in[it].curh - hn - in[it].gh;
        const floatx4 rc = in[it].curc - cn - in[it].gc;
        const long long ai = oa[it] + j;
        *reinterpret_cast<floatx4*>(a.gc + ai) = -rh;
        *reinterpret_cast<floatx4*>(a.gc + ai + H) = -rc;
        *reinterpret_cast<floatx4*>(a.uc + ai) = in[it].curh;
        *reinterpret_cast<floatx4*>(a.uc + ai + H) = in[it].curc;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          nrm += (double)rh[i] * (double)rh[i] + (double)rc[i] * (double)rc[i];
      } else {  // STEP_RHS
        *reinterpret_cast<floatx4*>(a.g + oi) = (in[it].curh - hn) + in[it].gh;
        *reinterpret_cast<floatx4*>(a.g + oi + H) = (in[it].curc - cn) + in[it].gc;
      }
    }
  }
}

// Rows = (level point, batch element); the contraction is h[R,H] . U[4H,H]^T on the fp32 MFMA
// tile core with four accumulator groups (one per gate), one workgroup per (row tile, column
// tile of the hidden width).
template <class C, int MODE>
__global__ __launch_bounds__(C::NT, C::NT > 256 ? 1 : C::MINWG) void lstm_step_kernel(PhiArgs a) {
  constexpr int LDSF =
      C::LDS_FLOATS > EpiStage<C>::FLOATS ? C::LDS_FLOATS : EpiStage<C>::FLOATS;
  __shared__ __attribute__((aligned(16))) float lds[LDSF];
  const int S = a.H, H = S / 2, B = a.B;
  const long long R = (long long)a.nk * B;
  long long rt;
  int ct;
  if (!xcd_tile(blockIdx.x, (R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN, rt, ct)) return;
  const long long m0 = rt * C::TM;
  const int n0 = ct * C::TN;
  const int tid = threadIdx.x;
  __shared__ LstmRow rowtab[C::TM];
  if (tid < C::TM) {
    long long r = m0 + tid;
    if (r >= R) r = R - 1;
    rowtab[tid] = lstm_row(a, r);
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
    arow[s] = a.u_in + (a.in.at(pt) * B + b) * S;       // h half of the state row
  }
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
  if (H % C::TK == 0)
    gemm_nt_tile<C, false>(acc, H, la, lb, Identity4(), Identity4(), lds);
  else
    gemm_nt_tile<C, true>(acc, H, la, lb, Identity4(), Identity4(), lds);

  double nrm = 0.0;
  lstm_tile_epilogue<C, MODE>(a, acc, rowtab, lds, m0, n0, R, nrm);
  if (MODE == STEP_RESID && a.norm) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_down(nrm, off, 64);
    if ((tid & 63) == 0) atomicAdd(a.norm, nrm);
  }
}

// Few rows (the coarsest level's serial propagation, a serial scan over a small batch): the
// vector-FMA form of skinny.h.  A workgroup owns a block of rows x CT hidden columns (4 CT
// weight rows); thread (row, column) applies the update to both halves of its element.
struct LstmEpiIn {
  float p[4], h, c, gh, gc, curh, curc;
};
template <int MODE>
__device__ inline LstmEpiIn lstm_epi_load(const PhiArgs& a, const LstmRow& ro, int j) {
  const int H = a.H / 2;
  LstmEpiIn e;
#pragma unroll
  for (int g = 0; g < 4; ++g) e.p[g] = a.P[ro.p + g * H + j] + a.b_h[g * H + j];
  e.h = a.u_in[ro.in + j];
  e.c = a.u_in[ro.in + H + j];
  e.gh = a.g ? a.g[ro.o + j] : 0.f;
  e.gc = a.g ? a.g[ro.o + H + j] : 0.f;
  e.curh = (MODE == STEP_RESID || MODE == STEP_RHS) ? a.u[ro.o + j] : 0.f;
  e.curc = (MODE == STEP_RESID || MODE == STEP_RHS) ? a.u[ro.o + H + j] : 0.f;
  return e;
}
template <int MODE>
__device__ inline void lstm_epi_finish(const PhiArgs& a, const LstmRow& ro, int j,
                                       const float (&s)[4], const LstmEpiIn& e, double& nrm) {
  const int H = a.H / 2;
  const LstmNew n = lstm_elem(a.gamma, a.propagator == PROP_LSTM_IMPLICIT, s[0] + e.p[0],
                              s[1] + e.p[1], s[2] + e.p[2], s[3] + e.p[3], e.h, e.c);
  const long long oi = ro.o + j;
  if (MODE == STEP_RELAX) {
    a.u[oi] = n.h + e.gh;
    a.u[oi + H] = n.c + e.gc;
  } else if (MODE == STEP_RESID) {
    const float rh = e.curh - n.h - e.gh, rc = e.curc - n.c - e.gc;
    const long long ai = ro.a + j;
    a.gc[ai] = -rh;
    a.gc[ai + H] = -rc;
    a.uc[ai] = e.curh;
    a.uc[ai + H] = e.curc;
    nrm += (double)rh * (double)rh + (double)rc * (double)rc;
  } else {  // STEP_RHS
    a.g[oi] = (e.curh - n.h) + e.gh;
    a.g[oi + H] = (e.curc - n.c) + e.gc;
  }
}

constexpr int LSTM_SK_ROWS = 32;   // rows per workgroup of the few-row step

template <int CT, int MODE>
__global__ __launch_bounds__(SK_MAXNT) void lstm_skinny_kernel(PhiArgs a,
                                                          int rows_block) {
  constexpr int NU = 4 * CT;
  constexpr int VP = sk_pow2_ceil(SK_RR * NU);
  __shared__ float red[(SK_MAXNT / 64) * VP];
  const int S = a.H, H = S / 2;
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
  LstmRow ero = {};
  LstmEpiIn ein = {};
  if (epi) {
    ero = lstm_row(a, r0 + tid / CT);
    e_j = j0 + tid % CT;
    ein = lstm_epi_load<MODE>(a, ero, e_j);
  }

  // rows beyond the block are clamped to its last row (their sums are never used)
  const float* hrow[SK_RR];
#pragma unroll
  for (int i = 0; i < SK_RR; ++i) {
    const int r = r0 + min(rg * SK_RR + i, rows_here - 1);
    const long long pt = (unsigned)r / (unsigned)a.B;
    const int b = r - (int)pt * a.B;
    hrow[i] = a.u_in + (a.in.at(pt) * a.B + b) * S;
  }
  const float* wrow[NU];
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const int g = u / CT, j = min(j0 + u % CT, H - 1);
    wrow[u] = (const float*)a.U + ((long long)g * H + j) * H;
  }
  float acc[SK_RR][NU];
  skinny_dot<NU, float>(acc, H, ks, ksl, wrow, [&](int i, int k) { return ldg4(hrow[i] + k); });
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
    float s[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) s[g] = skinny_sum<VP>(red, grp, base + g * CT + c, ksl);
    if (e == tid && epi) {
      lstm_epi_finish<MODE>(a, ero, e_j, s, ein, nrm);
    } else {   // more outputs than threads (tiny K only)
      const LstmRow ro = lstm_row(a, r0 + row);
      lstm_epi_finish<MODE>(a, ro, j, s, lstm_epi_load<MODE>(a, ro, j), nrm);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

// The few-row step on the matrix pipe (v_mfma_f32_16x16x4_f32), as the GRU's phi_fewrow_kernel: a
// workgroup owns 16 rows and four hidden columns, whose four gates are the 16 columns of the
// MFMA block; its waves split K (the h half of the state rows), each wave with all loads of its
// slice in flight before its first MFMA; the partial blocks meet in LDS and thread
// (row, column) applies the cell.  Lane l supplies A[i = l % 16][k = l / 16] and
// B[k = l / 16][j = l % 16]; result register v of lane l is D[4 (l / 16) + v][l % 16].
constexpr int LFR_NC = 4;      // hidden columns per workgroup
constexpr int LFR_KB = 8;      // blocks of sixteen k whose loads a wave keeps in flight
constexpr int LFR_MAXW = 8;    // waves per workgroup at most

template <int MODE>
__global__ __launch_bounds__(64 * LFR_MAXW) void lstm_fewrow_kernel(PhiArgs a, int kslice) {
  __shared__ float part[LFR_MAXW][16][17];
  const int S = a.H, H = S / 2;
  const int R = a.nk * a.B;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int nt = blockDim.x, nw = nt >> 6;
  const int li = lane & 15, kq = lane >> 4;
  const int j0 = blockIdx.x * LFR_NC;
  const int r0 = blockIdx.y * 16;
  const int rows_here = min(16, R - r0);

  // this thread's output element (if any): its operands are requested before the contraction
  const int n_out = rows_here * LFR_NC;
  const bool epi = tid < n_out && j0 + tid % LFR_NC < H;
  int e_j = 0;
  LstmRow ero = {};
  LstmEpiIn ein = {};
  if (epi) {
    ero = lstm_row(a, r0 + tid / LFR_NC);
    e_j = j0 + tid % LFR_NC;
    ein = lstm_epi_load<MODE>(a, ero, e_j);
  }

  // A: the h half of this lane's state row (rows beyond the block are clamped)
  const int r = r0 + min(li, rows_here - 1);
  const long long pt = (unsigned)r / (unsigned)a.B;
  const int b = r - (int)pt * a.B;
  const float* hrow = a.u_in + (a.in.at(pt) * a.B + b) * S;
  // B: weight row of this lane's MFMA column: gate li / 4, hidden column j0 + li % 4
  const float* urow = (const float*)a.U +
                      ((long long)(li / LFR_NC) * H + min(j0 + li % LFR_NC, H - 1)) * H;

  floatx4 acc = zero4(), acc1 = zero4();
  const int k_end = min(H, (wv + 1) * kslice);
  for (int kb = wv * kslice; kb < k_end; kb += 16 * LFR_KB) {
    floatx4 av[LFR_KB], bv[LFR_KB];
#pragma unroll
    for (int s = 0; s < LFR_KB; ++s) {
      const int k = kb + 16 * s + 4 * kq;
      const int kc = min(k, H - 4);                  // H is a multiple of 4
      av[s] = ldg4(hrow + kc);
      bv[s] = ldg4(urow + kc);
    }
    __builtin_amdgcn_sched_barrier(0);               // all loads in flight before the first wait
#pragma unroll
    for (int s = 0; s < LFR_KB; ++s) {
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
    const int row = e / LFR_NC, c = e % LFR_NC;
    const int j = j0 + c;
    if (j >= H) continue;
    float sg[4] = {0.f, 0.f, 0.f, 0.f};
    for (int w = 0; w < nw; ++w)
#pragma unroll
      for (int g = 0; g < 4; ++g) sg[g] += part[w][row][g * LFR_NC + c];
    if (e == tid && epi) {
      lstm_epi_finish<MODE>(a, ero, e_j, sg, ein, nrm);
    } else {   // more outputs than threads (one-wave workgroups only)
      const LstmRow ro = lstm_row(a, r0 + row);
      lstm_epi_finish<MODE>(a, ro, j, sg, lstm_epi_load<MODE>(a, ro, j), nrm);
    }
  }
  if (MODE == STEP_RESID && a.norm && nrm != 0.0) atomicAdd(a.norm, nrm);
}

static void launch_lstm_fewrow(const PhiArgs& a, hipStream_t s) {
  const int R = a.nk * a.B, H = a.H / 2;
  int nw = (H + 127) / 128;
  nw = nw < 1 ? 1 : (nw > LFR_MAXW ? LFR_MAXW : nw);
  const int kslice = ((H + nw - 1) / nw + 15) / 16 * 16;
  const dim3 grid((unsigned)((H + LFR_NC - 1) / LFR_NC), (unsigned)((R + 15) / 16));
  const dim3 block(64 * nw);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL(lstm_fewrow_kernel<STEP_RELAX>, grid, block, 0, s, a, kslice);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL(lstm_fewrow_kernel<STEP_RESID>, grid, block, 0, s, a, kslice);
  else
    hipLaunchKernelGGL(lstm_fewrow_kernel<STEP_RHS>, grid, block, 0, s, a, kslice);
}

template <int CT>
static void launch_lstm_skinny(const PhiArgs& a, dim3 grid, int rb, hipStream_t s) {
  int nt = sk_geom(rb, a.H / 2).nt;
  const dim3 block(nt);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL((lstm_skinny_kernel<CT, STEP_RELAX>), grid, block, 0, s, a, rb);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL((lstm_skinny_kernel<CT, STEP_RESID>), grid, block, 0, s, a, rb);
  else
    hipLaunchKernelGGL((lstm_skinny_kernel<CT, STEP_RHS>), grid, block, 0, s, a, rb);
}

// 128 rows x 64 hidden columns (x4 gates) as eight waves of 32 x 32 (x4): a wave's sums are
// dead once staged, which leaves the registers for the epilogue's ten operand vectors per item
typedef TileCfg<4, 2, 1, 1, 4> LstmBig;
typedef TileCfg<2, 2, 1, 1, 4> LstmMid;                  //  64 x 64
typedef TileCfg<1, 1, 1, 1, 4, 128, 1, 4> LstmSmall;     //  32 x 32, 4 waves splitting K

template <class C>
static void launch_lstm_cfg(const PhiArgs& a, hipStream_t s) {
  const long long R = (long long)a.nk * a.B;
  const int H = a.H / 2;
  dim3 grid((unsigned)xcd_grid((R + C::TM - 1) / C::TM, (H + C::TN - 1) / C::TN));
  dim3 block(C::NT);
  if (a.mode == STEP_RELAX)
    hipLaunchKernelGGL((lstm_step_kernel<C, STEP_RELAX>), grid, block, 0, s, a);
  else if (a.mode == STEP_RESID)
    hipLaunchKernelGGL((lstm_step_kernel<C, STEP_RESID>), grid, block, 0, s, a);
  else
    hipLaunchKernelGGL((lstm_step_kernel<C, STEP_RHS>), grid, block, 0, s, a);
}

// Up to 64 rows: the few-row kernel.  Above: tile shape by the number of workgroups it gives.
hipError_t launch_lstm_step(const PhiArgs& a, hipStream_t s) {
  if (a.nk <= 0) return hipSuccess;
  if (a.mode != STEP_RELAX && a.mode != STEP_RESID && a.mode != STEP_RHS)
    return hipErrorInvalidValue;
  const long long R = (long long)a.nk * a.B;
  const int H = a.H / 2;
  auto tiles = [&](int tm, int tn) { return ((R + tm - 1) / tm) * ((H + tn - 1) / tn); };
  prof_begin(9, s, R, a.mode);
  if (R <= 2 * SK_MAXROWS && H >= 16) {
    launch_lstm_fewrow(a, s);
  } else if (R <= 2 * SK_MAXROWS) {
    const int rb = R < LSTM_SK_ROWS ? (int)R : LSTM_SK_ROWS;
    const int nrb = (int)((R + rb - 1) / rb);
    const int ct = H * nrb >= 512 ? 2 : 1;
    dim3 grid((unsigned)((H + ct - 1) / ct), (unsigned)nrb);
    if (ct == 2)
      launch_lstm_skinny<2>(a, grid, rb, s);
    else
      launch_lstm_skinny<1>(a, grid, rb, s);
  } else if (tiles(LstmBig::TM, LstmBig::TN) >= 384)
    launch_lstm_cfg<LstmBig>(a, s);
  else if (R > 32 && tiles(LstmMid::TM, LstmMid::TN) >= 128)
    launch_lstm_cfg<LstmMid>(a, s);
  else
    launch_lstm_cfg<LstmSmall>(a, s);
  prof_end(9, 8.0 * (double)R * H * H, 32.0 * (double)R * H, s);
  return hipGetLastError();
}

}  // namespace mg
