// Internal declarations shared by the library's translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mgrit_gru.h"

namespace mg {

// Affine index of launch point i into an array of [*, B, width] blocks.
struct Idx {
  long long off, str;
  __host__ __device__ inline long long at(long long i) const { return off + i * str; }
};

enum StepMode {
  // out[o] = step(in) + g[o]   (Alg. 1 update; coarsest solve)
  STEP_RELAX = 0,
  // r = cur[o] - step(in) - g[o];  gc[a] = -r;  norm += r^2   (Alg. 2 lines 2-3)
  // forward: uc[a] = cur[o], the restricted iterate; adjoint: wc[a] = 0, the zero guess of the
  // error equation of a linear problem (see ff_cf for the exception in both)
  STEP_RESID = 1,
  // forward only: g[o] = cur[o] - step(in) + g[o]   (Eq. 11 right-hand side)
  STEP_RHS = 2,
  // forward only: adjoint coefficient vectors of the step
  STEP_KAPPA = 3,
  // forward only: STEP_RELAX that also leaves the coefficient vectors of the step it takes
  // (row = output point) in uc
  STEP_RELAX_KAPPA = 4,
  // forward only: STEP_RELAX from the coarse points of a level (first sub-step of an F-sweep)
  // that also evaluates the coarse level's step from the same inputs -- the contraction U h
  // does not depend on the step size -- and leaves  gc[a] = cur2 - step2(in), the first half
  // of the Eq. 11 right-hand side (STEP_RESID with resid_adds adds -r)
  STEP_RELAX_RHS = 5,
  // forward only: STEP_RELAX_KAPPA from the coarse points of level 0 that also leaves the
  // coefficient vectors of the coarse level's step from the same states (k_r, k_z, k_q, k_d;
  // row = coarse output point) in gc
  STEP_RELAX_KAPPA2 = 6,
  // forward only: STEP_RELAX from the coarse points of a level >= 1 that leaves the coarser
  // level's coefficient vectors like STEP_RELAX_KAPPA2
  STEP_RELAX_CK = 7
};

// One launch of the fused forward step  Phi_gamma(x, h) over nk level points.
struct PhiArgs {
  const void* U;       // [3H,H], float or bf16 (see bf16)
  const float* b_h;    // [3H]
  const float* P;      // [T,B,3H] input projection
  const float* u_in;   // state array the step reads from
  float* u;            // level state array (out for RELAX, cur for RESID/RHS)
  float* g;            // level right-hand side array (may be null = 0); RHS writes it
  float* uc;           // RESID: coarse state array   | KAPPA: coefficient array
  float* gc;           // RESID: coarse right-hand side array
  double* norm;        // RESID: sum of r^2 (may be null)
  Idx in, p, o, a;     // point indices: input state, projection row, out/cur/g, coarse
  int nk, B, H;
  int kappa_width;     // KAPPA: 4H or 5H floats per (point, b)
  float gamma;
  int propagator;
  int mode;
  int bf16;            // 1: U is bf16 and the contraction runs on the bf16 MFMA path
                       // 2: U is float; the tile kernels contract three-term bf16 operands
  const void* U3;      // bf16 == 2: the three bf16 terms of U, [3][3H,H]
  int zero_from;       // > 0: the input states of rows >= zero_from are all zero (tile kernels
                       // skip the contraction of tiles that start there; 0: nothing known)
  // STEP_RELAX_RHS: the second (coarse-level) evaluation of a row.  Its projection row and its
  // current coarse value sit at fixed element offsets from the row's own projection row
  // (index p) and output element (index o): both index pairs have the same stride.
  long long dp2;       // elements from the row's P row to the coarse step's P row
  long long do2;       // elements from the row's output row in u to the coarse point's row in u
  float gamma2;        // step size of the coarse level
  int resid_adds;      // STEP_RESID: gc[a] = gc[a] - r instead of -r (gc was prepared by
                       // STEP_RELAX_RHS)
  // STEP_RESID, ff_cf > 0: at coarse points whose index is ff_rem modulo ff_cf the coarse
  // array receives cur - r instead of cur.  Those are the points the coarse level's first
  // relaxation sub-step writes, and from the restricted iterate that sub-step gives
  // Phi_c(R u')_k + g_k = (R u')_k - (R r)_k by the definition of g (Eq. 11): no evaluation
  // of Phi is needed for it.
  int ff_cf, ff_rem;
  int one_term;        // bf16 == 1: the fp32 state operand goes to the MFMAs as one bf16 term
                       // (rounded) instead of two (hi + lo); tile kernels only
};

// One launch of the fused adjoint step  w_out = (dPhi/dh)^T w_in  over nk points.
struct AdjArgs {
  const void* UT;      // [H,3H] transposed recurrent weights, float or bf16
  const float* kap;    // coefficient array of this level, [*,B,kw]: k_r,k_z,k_q,k_d(,k_n)
  const float* w_in;   // adjoint array the step reads from
  float* w;            // level adjoint array (out / cur)
  float* g;            // level right-hand side (may be null)
  float* wc;           // RESID: coarse adjoint array
  float* gc;           // RESID: coarse right-hand side
  double* norm;
  Idx in, k, o, a;     // point indices: input adjoint, coefficient row, out/cur/g, coarse
  int nk, B, H, kw;
  int mode;
  int bf16;            // operand form, as in PhiArgs
  const void* UT3;     // bf16 == 2: the three bf16 terms of UT, [3][H,3H]
  int ff_cf, ff_rem;   // STEP_RESID: the coarse array wc receives the zero initial guess of the
                       // coarse error equation, except at the coarse points of index ff_rem
                       // modulo ff_cf (ff_cf > 0), which receive -r: the value the coarse level's
                       // first relaxation sub-step gives from that guess
  int one_term;        // as in PhiArgs (the operand kappa * w)
};

// Internal propagator code (beside the public MGRIT_PROP_* values): the forward-Euler
// step of the appendix's demonstration ODE (Eq. 17).  PhiArgs then reads U = A[H,H],
// P rows of width H (B d + b), gamma = step size of the level; b_h is unused.
constexpr int PROP_ODE_DEMO = 100;
// LSTM level step (kernels_lstm.hip), implicit in the decay terms / explicit.  PhiArgs then
// reads H = state width (2 x hidden width: h | c), U = U[4H_h, H_h], P rows of width 4H_h.
constexpr int PROP_LSTM_IMPLICIT = 101;
constexpr int PROP_LSTM_CLASSIC = 102;
__host__ __device__ inline bool prop_is_lstm(int p) {
  return p == PROP_LSTM_IMPLICIT || p == PROP_LSTM_CLASSIC;
}

// (dispatches to launch_ode_step for PROP_ODE_DEMO, to launch_lstm_step for the LSTM codes)
hipError_t launch_phi_step(const PhiArgs& a, hipStream_t s);
// modes STEP_RELAX, STEP_RESID, STEP_RHS; fp32 operands
hipError_t launch_ode_step(const PhiArgs& a, hipStream_t s);
// modes STEP_RELAX, STEP_RESID, STEP_RHS; fp32 operands
hipError_t launch_lstm_step(const PhiArgs& a, hipStream_t s);
hipError_t launch_adj_step(const AdjArgs& a, hipStream_t s);

// P[M,N] = X[M,K] W[N,K]^T + bias[N]
// X, W: float (bf16 = 0) or bf16 (bf16 = 1); bf16 = 2: X float, W the three bf16 terms
// [3][N,K] of the float weights
hipError_t launch_projection(const void* X, const void* W, const float* bias, float* P,
                             long long M, int N, int K, int bf16, hipStream_t s);
// UT[H,3H] = U[3H,H]^T; elements are 4 bytes (bf16 = 0) or 2 bytes
hipError_t launch_transpose(const void* U, void* UT, int rows, int cols, int bf16, hipStream_t s);

// Weight gradients (Alg. 3 gradient line) from the level-0 coefficients kap0[(T+1),B,5H]
// (row t = step t), the adjoint w[(T+1),B,H], the states h[(T+1),B,H] and x[T,B,D].
// part: scratch of grad_partial_floats(...) floats.
size_t grad_partial_floats(int T, int B, int D, int H, int bf16);
// x: float (bf16 = 0) or bf16 (bf16 = 1); one_term: as in PhiArgs (the wide bf16 kernel only;
// the narrow one keeps two terms)
hipError_t launch_param_grads(const float* kap0, const float* w, const float* h, const void* x,
                              float* dW, float* dU, float* db_i, float* db_h, float* part,
                              int T, int B, int D, int H, int bf16, int one_term, hipStream_t s);

// Input gradients dx[T,B,D] from the level-0 coefficients, the adjoint w and the
// transposed input weights WT[D,3H] (float, or bf16 with bf16 = 1, or its three bf16 terms
// [3][D,3H] with bf16 = 2).
hipError_t launch_input_grads(const float* kap0, const float* w, const void* WT, float* dx, int T,
                              int B, int D, int H, int bf16, int one_term, hipStream_t s);

// dst[t][i] (t = 0..2, bf16) = t-th term of src[i]: src = dst[0] + dst[1] + dst[2] exactly
// unless a term underflows; n a multiple of 4
hipError_t launch_split3(const float* src, void* dst, long long n, hipStream_t s);

hipError_t launch_fill_f64(double* p, long long n, double v, hipStream_t s);
// p[0..n) = 0; n a multiple of 4, p 16-byte aligned
hipError_t launch_zero_f32(float* p, long long n, hipStream_t s);
// dst[(d.off + i*d.str), :, :] = src[(s.off + i*s.str), :, :] for i < nk; blocks of `block` floats
hipError_t launch_copy_points(float* dst, const float* src, Idx d, Idx s, int nk, long long block,
                              hipStream_t st);
// dst[d.at(i)] += src[s.at(i)] for i < nk (blocks of `block` floats)
hipError_t launch_add_points(float* dst, const float* src, Idx d, Idx s, int nk, long long block,
                              hipStream_t st);
hipError_t launch_sqrt_to_float(const double* acc, float* out, int n, hipStream_t s);

// profiling brackets (see mgrit_gru_profile_enable)
// rows / mode describe the launch shape of a step kernel (0 / -1 where they do not apply)
void prof_begin(int kind, hipStream_t s, long long rows = 0, int mode = -1);
void prof_end(int kind, double flops, double bytes, hipStream_t s);

}  // namespace mg
