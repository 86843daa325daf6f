/*
 * mgrit_gru.h -- C ABI of the MI355X (gfx950) MGRIT-GRU library.
 *
 * Parallel-in-time forward and backward propagation of a one-layer GRU with
 * the multigrid-reduction-in-time (MGRIT) cycle of Moon & Cyr, "Parallel
 * Training of GRU Networks with a Multi-Grid Solver for Long Sequences"
 * (ICLR 2022), next to the serial time-step scan it replaces.
 *
 * Common conventions
 * ------------------
 * - Every data pointer is a DEVICE pointer unless the comment says "host".
 *   All arrays are dense row-major with the last index contiguous.
 * - x[T,B,D]: row t-1 holds x_t, t = 1..T.  State arrays have T+1 rows
 *   [(T+1),B,H]: row t holds h_t (or the adjoint w_t), row 0 is the initial
 *   condition (Sec. 3.1 notation; the paper fixes h_0 = 0, here it is passed).
 * - Parameters are those of the Classic GRU (Eq. 1), gates stacked in the
 *   order r, z, n:  W[3H,D] = (W_ir;W_iz;W_in), U[3H,H] = (W_hr;W_hz;W_hn),
 *   b_i[3H] = (b_ir;b_iz;b_in), b_h[3H] = (b_hr;b_hz;b_hn).  b_hn sits inside
 *   r*(W_hn h + b_hn), so the two bias sets cannot be merged.
 * - dtype MGRIT_F32: x, W, U are float.  MGRIT_BF16: x, W, U are bf16 (uint16
 *   bit patterns); biases, states, projections, accumulation and every output
 *   stay float.  The matrix pipe takes bf16 operands, so where a contraction's
 *   left operand is an fp32 state (U h, U^T(kappa w), the gradient sums) it is
 *   rounded to bf16 for that product only, as mixed-precision training does;
 *   the state that is stored, updated and returned stays fp32.
 *   MGRIT_BF16_STATE2: the same arguments, but the fp32 operand enters those
 *   products as two bf16 terms (hi + lo, 16 mantissa bits, twice the matrix
 *   work): results within ~1e-6 relative of fp64 arithmetic on the same bf16
 *   weights, where MGRIT_BF16 is within ~1e-2.  (The few-row steps of the
 *   coarsest level compute in fp32 on the bf16 weights under both.)
 *   MGRIT_F32_BF16X3: arguments exactly as for MGRIT_F32 and
 *   results to the same accuracy; the tile kernels carry each fp32 operand of
 *   a contraction as the sum of three bf16 terms (3 x 8 mantissa bits, the
 *   exponent range of fp32) and keep six of the nine term products, accumulated
 *   in fp32 on the bf16 matrix pipe, which is faster than the fp32 one.  The
 *   weights' term arrays live in the workspace (it is larger for this dtype)
 *   and are rebuilt by every call; H and D must be multiples of 8.
 * - Level l of the hierarchy has N_l = T / cf^l steps and step size cf^l
 *   (Sec. 3.3); `levels` counts the fine level (three levels over 128 steps
 *   with cf = 4 are grids of 128, 32 and 8 steps).  cf^(levels-1) must divide T.
 * - Ownership: the caller owns every buffer including the workspace.  The
 *   library never allocates or frees device memory, and the compute entry
 *   points never synchronise the device: all their work is enqueued on
 *   `stream` (a hipStream_t passed as void*; NULL is the default stream).  The
 *   only calls that wait are mgrit_gru_profile_read / _read_shape, which
 *   synchronise on the timing events they report.  Outputs are overwritten,
 *   never accumulated.
 * - Errors: every entry point returns 0 on success or a negative MGRIT_E_*
 *   code.  Arguments are validated on the host before anything is launched:
 *   with every code except MGRIT_E_LAUNCH a failing call has launched nothing
 *   and all buffers are untouched.  MGRIT_E_LAUNCH is returned from the middle
 *   of the work when the HIP runtime refuses a launch; outputs and workspace are
 *   then undefined.  (An error state left on the calling thread by earlier,
 *   unrelated HIP work is cleared at entry and not reported.)  No exception
 *   crosses the ABI.  mgrit_gru_strerror() names a code.
 * - Calls that share a workspace must be ordered on one stream.
 * - resnorm_out values are sums of squares accumulated with floating-point
 *   atomics in double precision: reproducible to about 1e-15 relative, not
 *   bit for bit; every other output is bitwise reproducible.
 */
#ifndef MGRIT_GRU_H
#define MGRIT_GRU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define MGRIT_API __attribute__((visibility("default")))
#else
#define MGRIT_API
#endif

enum {
  MGRIT_OK = 0,
  MGRIT_E_NULL = -1,        /* a required pointer is NULL */
  MGRIT_E_SIZE = -2,        /* T, B, D, H, cf, levels or iters out of range */
  MGRIT_E_HIERARCHY = -3,   /* cf^(levels-1) does not divide T */
  MGRIT_E_ENUM = -4,        /* unknown propagator / dtype / fine_relax / flags */
  MGRIT_E_WORKSPACE = -5,   /* workspace smaller than mgrit_gru_workspace_bytes */
  MGRIT_E_ALIGN = -6,       /* H or D not a multiple of 4 (MGRIT_F32) / 8 (other dtypes),
                               or a pointer not 16-byte aligned */
  MGRIT_E_LAUNCH = -7,      /* the HIP runtime refused a launch */
  MGRIT_E_UNSUPPORTED = -8, /* a valid request this build has no kernel for */
  MGRIT_E_STATE = -9        /* MGRIT_REUSE_PROJECTION / MGRIT_REUSE_COEFFS, but the library's
                               host-side record of this workspace pointer says the projection
                               / coefficient vectors of another problem (other sizes, hierarchy,
                               dtype, propagator, x / W / b_i / h arrays), or none, were left
                               there.  The record cannot see memory overwritten by others or
                               arrays changed in place: that part stays the caller's promise */
};

enum { MGRIT_PROP_IMPLICIT = 0,   /* Eq. 16, the paper's propagator on all levels */
       MGRIT_PROP_CLASSIC = 1 };  /* Eq. 3 (explicit Euler; Classic GRU when step = 1) */
enum { MGRIT_F32 = 0, MGRIT_BF16 = 1, MGRIT_F32_BF16X3 = 2, MGRIT_BF16_STATE2 = 3 };

/* flags */
enum {
  /* The workspace already holds the input projection of these x, W, b_i (left
   * there by an earlier call with the same sizes and dtype): skip recomputing
   * it.  The paper likewise computes per-step input features once and reuses
   * them on coarse grids and in back-propagation (Appendix A.3.2). */
  MGRIT_REUSE_PROJECTION = 1,
  /* Forward calls (mgrit_gru_forward with iters >= 1, gru_serial_scan): while the
   * closing F-relaxation of the last cycle (Alg. 2 line 6; every step of the
   * serial scan) writes the final states, also leave in the workspace the
   * coefficient vectors of the transposed Jacobian of each step it takes
   * (Appendix A.2), which the adjoint solve would otherwise recompute; with
   * more than one level its first sub-step, which starts from the coarse points,
   * leaves the vectors of every step of level 1 as well (same states, same
   * recurrent contraction, the coarse step size and inputs), and so do the
   * closing relaxations of the coarse levels for the level below them, except
   * for the coarsest level.  (A
   * serial scan over 64 or fewer batch rows leaves none: there one pass over
   * all steps in the backward call is cheaper; the backward call knows.) */
  MGRIT_KEEP_COEFFS = 2,
  /* Backward calls: the workspace holds what a forward call with
   * MGRIT_KEEP_COEFFS left there, for the same sizes, hierarchy, dtype,
   * propagator and workspace pointer, and the states h passed in are the ones
   * that call returned: only the steps it did not cover (those of level 0
   * into the coarse points, and the coarsest level beyond level 1) are
   * linearised again.  A backward call leaves the vectors of every step, so a
   * further backward call on the same problem may reuse them too.  Checked
   * against the host-side record of the workspace (MGRIT_E_STATE), like
   * MGRIT_REUSE_PROJECTION. */
  MGRIT_REUSE_COEFFS = 4,
  /* mgrit_gru_backward: rows 0..T-1 of w_inout are zero on entry (the initial
   * guess of Alg. 3).  The adjoint recurrence is linear and homogeneous, so in
   * the first cycle everything below the last intervals is still zero when the
   * relaxation, residual and right-hand-side passes reach it; with this flag
   * those passes skip the rows whose result is known to be zero (the zeros are
   * written where a coarse level needs them).  The iterate returned is the same
   * up to rounding (a pass over fewer rows may run in another kernel form, which
   * adds in another order).  With mgrit_gru_backward_steps the flag declares in
   * addition that rows 0..T-1 of dL_dh are zero (the top layer of a stack whose
   * loss reads h_T only, called through this entry point for its dx); with a
   * loss term on earlier states it must not be set.  Ignored by the serial
   * entry points. */
  MGRIT_ZERO_ADJOINT_GUESS = 8,
  /* mgrit_gru_forward: rows 1..T of h_inout are zero on entry (the initial guess
   * of Alg. 3).  The first sub-step of the first relaxation then starts from
   * zero states everywhere but in the first interval, and its recurrent
   * contraction U h is skipped where h is zero (the sums are exactly zero
   * either way: the iterate is the same, bit for bit).  Ignored by the serial
   * scan. */
  MGRIT_ZERO_STATE_GUESS = 16
};

typedef struct {
  int32_t T, B, D, H;   /* sequence length, batch, input width, hidden width */
  int32_t cf;           /* coarsening factor (Sec. 3.1), >= 1 */
  int32_t levels;       /* grid levels including the fine one, >= 1; 1 = serial */
  int32_t iters;        /* MGRIT cycles applied by this call (Remark 1), >= 0 */
  int32_t fine_relax;   /* level-0 relaxation in Alg. 2 line 1: 0 = F, 1 = FCF
                           (Eq. 8); coarser levels always use FCF */
  int32_t propagator;   /* MGRIT_PROP_* */
  int32_t dtype;        /* MGRIT_F32 / MGRIT_BF16 / MGRIT_F32_BF16X3 / MGRIT_BF16_STATE2 */
  int32_t flags;        /* 0 or an OR of the flags above */
} mgrit_gru_cfg;

/* Bytes of device workspace one call needs (host-only computation).  The same
 * workspace serves every entry point; its first bytes hold the input
 * projection P[T,B,3H] (float) so that MGRIT_REUSE_PROJECTION works across
 * calls.  cfg: host pointer.  bytes: host pointer, receives the size. */
MGRIT_API int mgrit_gru_workspace_bytes(const mgrit_gru_cfg* cfg, size_t* bytes);

/* Serial forward propagation h_t = Phi_1(x_t, h_{t-1}), t = 1..T: the solution
 * of f(h) = 0 in Eq. 4, with Phi the step selected by cfg->propagator (Eq. 16 or
 * Eq. 3).  cf, levels, iters, fine_relax are ignored.
 *   h0[B,H] in; h_out[(T+1),B,H] out (row 0 receives h0). */
MGRIT_API int gru_serial_scan(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                    const float* b_i, const float* b_h, const void* x,
                    const float* h0, float* h_out,
                    void* workspace, size_t workspace_bytes, void* stream);

/* MGRIT forward propagation: cfg->iters applications of MGProp (Alg. 2, made
 * recursive over cfg->levels as in Remark 2, coarse equation Eq. 11, coarsest
 * level solved by serial propagation) to the iterate in h_inout.
 *   h_inout[(T+1),B,H]: initial guess in (Alg. 3 uses zeros), iterate out; row 0
 *     is overwritten with h0.
 *   resnorm_out[iters] (device, may be NULL): 2-norm of the level-0 residual
 *     (Eq. 4) at the coarse points after the relaxation of Alg. 2 line 1, one
 *     value per cycle (the residual at F-points is zero there). */
MGRIT_API int mgrit_gru_forward(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                      const float* b_i, const float* b_h, const void* x,
                      const float* h0, float* h_inout, float* resnorm_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Serial back-propagation through time for a loss on h_T (discrete adjoint of
 * the step, Appendix A.2): w_T = dL_dhT, w_{t-1} = (dPhi_1/dh)^T(x_t,h_{t-1}) w_t,
 * and the parameter gradients g = sum_t w_t dh_t/dTheta (Alg. 3, gradient line).
 *   h[(T+1),B,H] in: forward states (linearisation points).
 *   w_out[(T+1),B,H] out; row 0 is dL/dh_0.
 *   dW[3H,D], dU[3H,H], db_i[3H], db_h[3H] out (float). */
MGRIT_API int gru_serial_scan_backward(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                             const float* b_i, const float* b_h, const void* x,
                             const float* h, const float* dL_dhT, float* w_out,
                             float* dW, float* dU, float* db_i, float* db_h,
                             void* workspace, size_t workspace_bytes, void* stream);

/* MGRIT back-propagation: cfg->iters applications of MGBackProp, i.e. the same
 * cycle run on the adjoint recurrence in reversed time (Appendix A.1 last
 * paragraph, A.2 last paragraph; Alg. 3 backward block), each level step being
 * the transposed Jacobian of that level's forward step linearised at the given
 * forward iterate h; then the parameter gradients from the final w.  (The
 * adjoint recurrence is linear: the coarse equations of the cycle are solved
 * for the error, which gives the iterates of the Eq. 11 form up to rounding.)
 *   w_inout[(T+1),B,H]: initial guess in (Alg. 3 uses zeros), iterate out; row T
 *     is overwritten with dL_dhT.
 *   resnorm_out[iters] (device, may be NULL): as in mgrit_gru_forward, for the
 *     adjoint level-0 equation.
 *   dW, dU, db_i, db_h: as in gru_serial_scan_backward; any of them may be NULL
 *     only if all four are NULL (then no gradients are formed). */
MGRIT_API int mgrit_gru_backward(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                       const float* b_i, const float* b_h, const void* x,
                       const float* h, const float* dL_dhT, float* w_inout,
                       float* resnorm_out,
                       float* dW, float* dU, float* db_i, float* db_h,
                       void* workspace, size_t workspace_bytes, void* stream);

/* The two back-propagations above for a loss that depends on every state, and
 * with the gradient with respect to the inputs: what a stack of GRU layers
 * (Sec. 4: two layers in every experiment) needs, layer j+1 reading the states
 * of layer j as its input sequence and handing dL/dx back as layer j's loss term.
 *   dL_dh[(T+1),B,H] in (device, 16-byte aligned): row t holds the direct
 *     derivative of the loss with respect to h_t (row 0: h_0).  The adjoint
 *     recurrence of Appendix A.2 gains it as a source term,
 *         w_T = dL_dh[T],   w_{t-1} = (dPhi_1/dh)^T(x_t,h_{t-1}) w_t + dL_dh[t-1],
 *     which is the right-hand side of the level-0 equation of the cycle; coarse
 *     levels receive it through the restriction of Eq. 11 like any residual.
 *     A loss on h_T alone is the array that is zero except for row T.
 *   dx[T,B,D] out (device, float, may be NULL): row t-1 receives
 *     dL/dx_t = (dPhi_1/dx)^T(x_t,h_{t-1}) w_t, formed from the final w like the
 *     parameter gradients (Alg. 3, gradient line).
 * All other arguments, and the error behaviour, are those of
 * gru_serial_scan_backward / mgrit_gru_backward. */
MGRIT_API int gru_serial_scan_backward_steps(const mgrit_gru_cfg* cfg, const void* W,
                             const void* U, const float* b_i, const float* b_h, const void* x,
                             const float* h, const float* dL_dh, float* w_out,
                             float* dW, float* dU, float* db_i, float* db_h, float* dx,
                             void* workspace, size_t workspace_bytes, void* stream);
MGRIT_API int mgrit_gru_backward_steps(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                       const float* b_i, const float* b_h, const void* x,
                       const float* h, const float* dL_dh, float* w_inout,
                       float* resnorm_out,
                       float* dW, float* dU, float* db_i, float* db_h, float* dx,
                       void* workspace, size_t workspace_bytes, void* stream);

/* mgrit_gru_forward for callers that cannot allocate device memory or pass a
 * workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the workspace is a fixed array of
 * MGRIT_STATIC_SCRATCH_BYTES inside the library's code object, one copy per
 * GPU, held until the process ends.  Same arguments (minus workspace), same
 * kernels, same results as mgrit_gru_forward.
 *   - cfg->flags: 0 or MGRIT_ZERO_STATE_GUESS (MGRIT_E_UNSUPPORTED otherwise:
 *     nothing is kept in or reused from this workspace across calls).
 *   - MGRIT_E_WORKSPACE if mgrit_gru_workspace_bytes(cfg) exceeds
 *     MGRIT_STATIC_SCRATCH_BYTES; checked before anything is launched.
 *   - Calls no hipMalloc / hipFree / event or stream creation; with profiling
 *     enabled its launches are not bracketed.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one
 *     GPU (different streams or threads) race.  Everything the cycle reads from
 *     the array it has written earlier in the same call. */
#define MGRIT_STATIC_SCRATCH_BYTES (64u << 20)
MGRIT_API int mgrit_gru_forward_static(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                      const float* b_i, const float* b_h, const void* x,
                      const float* h0, float* h_inout, float* resnorm_out, void* stream);

/* A second propagator behind the same forward cycle: the demonstration ODE of the
 * appendix "Why does MGRIT work?" (Eq. 17),
 *     dh/dt = -h/2 + sigmoid(A h + B d(t) + b),
 * forward propagation only, as in the paper.  The appendix does not print the
 * discretisation; here a step is forward Euler over one data sample,
 *     Phi_dt(h_{t-1}; d_t) = h_{t-1} + dt (-h_{t-1}/2 + sigmoid(A h_{t-1} + B d_t + b)),
 * and level l of the hierarchy uses the step size cf^l dt with the data of its own
 * points (the rule of Sec. 3.3).
 *   cfg: T, B, D, H, cf, levels, iters, fine_relax as for the GRU entry points;
 *     dtype must be MGRIT_F32 and flags 0 (MGRIT_E_UNSUPPORTED otherwise);
 *     propagator is not read.  dt: level-0 step size, finite and > 0.
 *   A[H,H], Bw[H,D], b[H], d[T,B,D] (row t-1 holds d_t), h0[B,H]: device, float.
 *   h_out / h_inout[(T+1),B,H], resnorm_out[iters]: as for gru_serial_scan and
 *     mgrit_gru_forward.
 *   workspace: mgrit_gru_workspace_bytes(cfg) bytes serve these calls too. */
MGRIT_API int ode_serial_scan(const mgrit_gru_cfg* cfg, float dt, const float* A,
                    const float* Bw, const float* b, const float* d,
                    const float* h0, float* h_out,
                    void* workspace, size_t workspace_bytes, void* stream);
MGRIT_API int mgrit_ode_forward(const mgrit_gru_cfg* cfg, float dt, const float* A,
                      const float* Bw, const float* b, const float* d,
                      const float* h0, float* h_inout, float* resnorm_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* A third propagator behind the same forward cycle: an LSTM layer, the extension the
 * paper's conclusion names.  The paper gives no equations for it; the step here is derived
 * the way Sec. 3.3 derives the Implicit GRU.  With the gates i, f, o = sigmoid(.), g = tanh(.)
 * of W x_t + b_i + U h_{t-1} + b_h (stacked in the order i, f, g, o), the standard cell
 * c_t = f c_{t-1} + i g, h_t = o tanh(c_t) is a forward-Euler step of size 1 of
 *     dc/dt = -(1 - f) c + i g,      dh/dt = -h + o tanh(c),
 * and a level step of size gamma is, with the decay terms taken implicitly
 * (cfg->propagator = MGRIT_PROP_IMPLICIT),
 *     c' = (c + gamma i g) / (1 + gamma (1 - f)),    h' = (h + gamma o tanh(c')) / (1 + gamma),
 * or explicitly (MGRIT_PROP_CLASSIC; gamma = 1 is the standard LSTM cell)
 *     c' = c + gamma (-(1 - f) c + i g),             h' = h + gamma (-h + o tanh(c')).
 * Level l uses gamma = cf^l and the inputs of its own points (Sec. 3.1, 3.3).  Forward
 * propagation only.
 *   cfg: as for the GRU entry points, H = hidden width; dtype must be MGRIT_F32 and flags 0
 *     (MGRIT_E_UNSUPPORTED otherwise).
 *   W[4H,D], U[4H,H], b_i[4H], b_h[4H], x[T,B,D]: device, float.
 *   The state of the time integration is the pair (h, c): u0[B,2H] and the rows of
 *   u_out / u_inout[(T+1),B,2H] hold h in columns 0..H-1 and c in columns H..2H-1.
 *   resnorm_out[iters]: 2-norm of the level-0 residual over both halves, as in mgrit_gru_forward.
 *   workspace: mgrit_lstm_workspace_bytes(cfg) bytes (host-only computation). */
MGRIT_API int mgrit_lstm_workspace_bytes(const mgrit_gru_cfg* cfg, size_t* bytes);
MGRIT_API int lstm_serial_scan(const mgrit_gru_cfg* cfg, const float* W, const float* U,
                    const float* b_i, const float* b_h, const float* x,
                    const float* u0, float* u_out,
                    void* workspace, size_t workspace_bytes, void* stream);
MGRIT_API int mgrit_lstm_forward(const mgrit_gru_cfg* cfg, const float* W, const float* U,
                      const float* b_i, const float* b_h, const float* x,
                      const float* u0, float* u_inout, float* resnorm_out,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Name of an error code (host string with static storage). */
MGRIT_API const char* mgrit_gru_strerror(int code);

/* Kernel timing for benchmarks.  While enabled, every launch of the fused
 * step kernels (the dominant kernels: recurrent contraction + gates) is
 * bracketed by HIP events on the launch stream.  mgrit_gru_profile_read
 * synchronises those events and returns, per kernel class, the number of
 * launches, their summed duration in milliseconds and their summed
 * algorithmic flops and bytes; it then clears what it returned.  Event objects are
 * host-side and created on demand; nothing here touches device memory.  Switching
 * profiling on starts an empty record; the record holds at most 2^18 launches
 * (later ones run unbracketed until a read makes room).
 *   kind: 0 = forward step (Phi) on MFMA tiles, 1 = adjoint step (Phi^T) on MFMA tiles,
 *         2 = projection GEMM, 3 = weight-gradient GEMMs, 4 / 5 = forward / adjoint step
 *         in the few-row form used by the serial scan and the coarsest-level solve,
 *         6 = input-gradient GEMM, 7 = point copies (coarse-grid correction, terminal and
 *         initial conditions), 8 = step of the demonstration ODE (tile and few-row forms),
 *         9 = LSTM step (tile and few-row forms).
 * All out-pointers are host pointers. */
MGRIT_API int mgrit_gru_profile_enable(int on);
MGRIT_API int mgrit_gru_profile_read(int kind, int64_t* launches, double* ms,
                           double* flops, double* bytes);
/* The same for one launch shape of a step kernel class (kind 0, 1, 4, 5, 8, 9): only the
 * launches that advance `rows` rows (level points x batch) in epilogue mode `mode`
 * (0 = relaxation update, 1 = residual + restriction, 2 = coarse right-hand side,
 * 3 = coefficients, 4 = relaxation update that keeps the coefficients, 5 = relaxation
 * update from the coarse points that also evaluates the coarse level's step, 6 = mode 4
 * that also leaves the coefficients of level 1, 7 = mode 0 that leaves the coefficients
 * of the next level; + 16 for a
 * forward launch that skips the contraction of zero-input tiles, whose flops count
 * the rows it contracts only); a negative value matches any.  Records that do not
 * match stay for later reads. */
MGRIT_API int mgrit_gru_profile_read_shape(int kind, int64_t rows, int mode,
                           int64_t* launches, double* ms, double* flops, double* bytes);

#ifdef __cplusplus
}
#endif
#endif /* MGRIT_GRU_H */
