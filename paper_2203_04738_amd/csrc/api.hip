// C ABI of the MGRIT-GRU library: argument validation, workspace layout and the
// host-side level drivers that enqueue the kernels of one MGRIT cycle
// (Alg. 2 of the paper, recursive per Remark 2) for the forward recurrence and
// for its adjoint in reversed time.
#include <cstdint>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "common.h"

// Workspace of mgrit_gru_forward_static: one array per GPU, held from the moment the library's
// code object is loaded on that GPU until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels and fills take the address that call returns.
static __device__ __align__(256) unsigned char scratch[MGRIT_STATIC_SCRATCH_BYTES];

namespace mg {

constexpr int MAX_LEVELS = 24;
constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[MAX_DEVICES] = {};   // [device]: address of `scratch` on that GPU

// Address of the current device's copy of `scratch` (looked up once per device).
static int static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return MGRIT_E_LAUNCH;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MGRIT_E_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MGRIT_OK;
}

// ---------------------------------------------------------------------------
// profiling brackets
// ---------------------------------------------------------------------------
struct ProfRec {
  int kind, mode;
  long long rows;
  hipEvent_t e0, e1;
  double flops, bytes;
  bool open;           // begun, end not yet recorded
};
static bool g_prof = false;
static std::mutex g_prof_mu;
static std::vector<ProfRec> g_recs;
// Launches recorded while profiling is on and nobody reads: beyond this many the record stops
// growing (further launches run unbracketed) until a read or mgrit_gru_profile_enable clears it.
constexpr size_t MAX_PROF_RECS = 1u << 18;
// set for the duration of a call that must create no runtime objects (the entry point that
// allocates nothing): its launches are never bracketed
static thread_local bool t_no_prof = false;

void prof_begin(int kind, hipStream_t s, long long rows, int mode) {
  if (!g_prof || t_no_prof) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_recs.size() >= MAX_PROF_RECS) return;
  ProfRec r;
  r.kind = kind;
  r.rows = rows;
  r.mode = mode;
  r.flops = r.bytes = 0;
  r.open = true;
  if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return;
  (void)hipEventRecord(r.e0, s);
  g_recs.push_back(r);
}

void prof_end(int kind, double flops, double bytes, hipStream_t s) {
  if (!g_prof || t_no_prof) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (g_recs.empty() || g_recs.back().kind != kind || !g_recs.back().open) return;
  g_recs.back().open = false;
  g_recs.back().flops = flops;
  g_recs.back().bytes = bytes;
  (void)hipEventRecord(g_recs.back().e1, s);
}

// ---------------------------------------------------------------------------
// validation and workspace layout (host only)
// ---------------------------------------------------------------------------
struct Layout {
  int L;
  long long N[MAX_LEVELS];        // steps on level l
  long long S[MAX_LEVELS];        // step size cf^l
  size_t P;                       // offsets in bytes
  size_t u[MAX_LEVELS], g[MAX_LEVELS];
  size_t tmp;                     // cf == 1 only: Jacobi scratch for the C-sweep
  size_t norm;
  size_t kap[MAX_LEVELS];
  size_t UT, WT, part;
  size_t U3, UT3, W3;             // MGRIT_F32_BF16X3: three-term bf16 copies of U, U^T and
                                  // W (or W^T, once the projection is done)
  size_t total;
};

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

// Operand form handed to the kernels: 0 fp32, 1 bf16 inputs and weights, 2 three bf16 terms per
// fp32 operand; both bf16 dtypes store alike and differ in how the tile kernels carry the fp32
// state operand (one bf16 term, or two with MGRIT_BF16_STATE2).
static int kform(int dtype) { return dtype == MGRIT_BF16_STATE2 ? 1 : dtype; }
static int one_term(int dtype) { return dtype == MGRIT_BF16 ? 1 : 0; }

static int check_cfg(const mgrit_gru_cfg* c, bool need_hierarchy) {
  if (!c) return MGRIT_E_NULL;
  if (c->T < 1 || c->B < 1 || c->D < 1 || c->H < 1) return MGRIT_E_SIZE;
  if ((long long)c->T * c->B > (1LL << 30)) return MGRIT_E_SIZE;
  if (c->iters < 0) return MGRIT_E_SIZE;
  if (c->propagator != MGRIT_PROP_IMPLICIT && c->propagator != MGRIT_PROP_CLASSIC)
    return MGRIT_E_ENUM;
  if (c->dtype != MGRIT_F32 && c->dtype != MGRIT_BF16 && c->dtype != MGRIT_F32_BF16X3 &&
      c->dtype != MGRIT_BF16_STATE2)
    return MGRIT_E_ENUM;
  if (c->flags & ~(MGRIT_REUSE_PROJECTION | MGRIT_KEEP_COEFFS | MGRIT_REUSE_COEFFS |
                   MGRIT_ZERO_ADJOINT_GUESS | MGRIT_ZERO_STATE_GUESS))
    return MGRIT_E_ENUM;
  if (need_hierarchy) {
    if (c->cf < 1 || c->levels < 1 || c->levels > MAX_LEVELS) return MGRIT_E_SIZE;
    if (c->fine_relax != 0 && c->fine_relax != 1) return MGRIT_E_ENUM;
    long long s = 1;
    for (int l = 1; l < c->levels; ++l) {
      s *= c->cf;
      if (s > c->T) return MGRIT_E_HIERARCHY;
    }
    if (c->T % s != 0) return MGRIT_E_HIERARCHY;
  }
  const int mult = c->dtype == MGRIT_F32 ? 4 : 8;
  if (c->H % mult != 0 || c->D % mult != 0) return MGRIT_E_ALIGN;
  return MGRIT_OK;
}

static int make_layout(const mgrit_gru_cfg* c, Layout* lay) {
  std::memset(lay, 0, sizeof(*lay));
  const int L = c->levels < 1 ? 1 : c->levels;
  lay->L = L;
  long long s = 1;
  for (int l = 0; l < L; ++l) {
    lay->S[l] = s;
    lay->N[l] = c->T / s;
    s *= c->cf;
  }
  const size_t BH = (size_t)c->B * c->H * sizeof(float);
  size_t off = 0;
  lay->P = off;
  off = align_up(off + (size_t)c->T * c->B * 3 * c->H * sizeof(float));
  for (int l = 1; l < L; ++l) {
    lay->u[l] = off;
    off = align_up(off + (size_t)(lay->N[l] + 1) * BH);
    lay->g[l] = off;
    off = align_up(off + (size_t)(lay->N[l] + 1) * BH);
  }
  lay->tmp = off;
  if (c->cf == 1 && L > 1) off = align_up(off + (size_t)(c->T + 1) * BH);
  for (int l = 0; l < L; ++l) {
    lay->kap[l] = off;
    off = align_up(off + (size_t)(lay->N[l] + 1) * BH * (l == 0 ? 5 : 4));
  }
  lay->UT = off;
  off = align_up(off + (size_t)3 * c->H * c->H * sizeof(float));
  lay->WT = off;
  off = align_up(off + (size_t)3 * c->H * c->D * sizeof(float));
  lay->part = off;
  off = align_up(off + grad_partial_floats(c->T, c->B, c->D, c->H, kform(c->dtype)) * sizeof(float));
  if (c->dtype == MGRIT_F32_BF16X3) {
    lay->U3 = off;
    off = align_up(off + (size_t)3 * 3 * c->H * c->H * 2);
    lay->UT3 = off;
    off = align_up(off + (size_t)3 * 3 * c->H * c->H * 2);
    lay->W3 = off;
    off = align_up(off + (size_t)3 * 3 * c->H * c->D * 2);
  }
  // last, because its size depends on iters: everything before it sits at the same
  // offset in every call with the same sizes and hierarchy (projection and coefficient
  // arrays can be reused across calls)
  lay->norm = off;
  off = align_up(off + (size_t)(c->iters > 0 ? c->iters : 1) * sizeof(double));
  lay->total = off;
  return MGRIT_OK;
}

static bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

#define CHECK_HIP(expr)                          \
  do {                                           \
    if ((expr) != hipSuccess) return MGRIT_E_LAUNCH; \
  } while (0)

// ---------------------------------------------------------------------------
// what a workspace holds (host-side record; no device read, no synchronisation)
// ---------------------------------------------------------------------------
// MGRIT_REUSE_PROJECTION and MGRIT_REUSE_COEFFS are promises about the contents of the
// caller's workspace.  The call that leaves the projection / the coefficient vectors there
// notes, under the workspace pointer, the problem they belong to; a call that asks to reuse
// them is refused (MGRIT_E_STATE, before any launch) unless its own problem matches.  The
// record cannot see a workspace that was overwritten by something else than this library, nor
// input arrays whose contents changed in place: those stay the caller's promise.
struct WsRecord {
  bool have_proj = false, have_coeffs = false;
  // projection: sizes, operand form, row width (3H, or H for the demonstration ODE) and the
  // arrays it was computed from
  int pT = 0, pB = 0, pD = 0, pH = 0, pdtype = 0, pwidth = 0;
  const void *px = nullptr, *pW = nullptr, *pbi = nullptr;
  // coefficient vectors: the configuration of the forward call that kept them and the state
  // array they were linearised at
  mgrit_gru_cfg ccfg{};
  bool cserial = false;
  const void* ch = nullptr;
};
static std::mutex g_ws_mu;
static std::unordered_map<const void*, WsRecord> g_ws;
constexpr size_t MAX_WS_RECORDS = 1024;   // beyond that the table starts over (reuse is then
                                          // refused until the producing call runs again)

static WsRecord ws_record_get(const void* ws) {
  std::lock_guard<std::mutex> lk(g_ws_mu);
  auto it = g_ws.find(ws);
  return it == g_ws.end() ? WsRecord{} : it->second;
}
static void ws_record_put(const void* ws, const WsRecord& r) {
  std::lock_guard<std::mutex> lk(g_ws_mu);
  if (g_ws.size() >= MAX_WS_RECORDS && g_ws.find(ws) == g_ws.end()) g_ws.clear();
  g_ws[ws] = r;
}

static bool proj_matches(const WsRecord& r, const mgrit_gru_cfg& c, int width, const void* x,
                         const void* W, const void* b_i) {
  return r.have_proj && r.pT == c.T && r.pB == c.B && r.pD == c.D && r.pH == c.H &&
         r.pdtype == c.dtype && r.pwidth == width && r.px == x && r.pW == W && r.pbi == b_i;
}
static void proj_note(WsRecord& r, const mgrit_gru_cfg& c, int width, const void* x,
                      const void* W, const void* b_i) {
  // a projection of other sizes moves every later array of the layout
  if (r.pT != c.T || r.pB != c.B || r.pD != c.D || r.pH != c.H || r.pdtype != c.dtype)
    r.have_coeffs = false;
  r.have_proj = true;
  r.pT = c.T; r.pB = c.B; r.pD = c.D; r.pH = c.H;
  r.pdtype = c.dtype; r.pwidth = width;
  r.px = x; r.pW = W; r.pbi = b_i;
}
static bool coeffs_match(const WsRecord& r, const mgrit_gru_cfg& c, bool serial, const void* h) {
  if (!r.have_coeffs || r.cserial != serial || r.ch != h) return false;
  const mgrit_gru_cfg& k = r.ccfg;
  if (k.T != c.T || k.B != c.B || k.D != c.D || k.H != c.H || k.dtype != c.dtype ||
      k.propagator != c.propagator)
    return false;
  return serial || (k.cf == c.cf && k.levels == c.levels);
}

// ---------------------------------------------------------------------------
// forward drivers
// ---------------------------------------------------------------------------
struct FwdCtx {
  const mgrit_gru_cfg* c;
  const Layout* lay;
  const void *U, *U3;
  const float *b_h, *P;
  float* ul[MAX_LEVELS];
  float* gl[MAX_LEVELS];
  float* tmp;
  double* norm;     // accumulator of the current cycle (may be null)
  float* emit_kap;  // level-0 coefficient array the closing relaxation also fills (or null)
  float* emit_kapl[MAX_LEVELS];  // [l]: coefficient array of level l >= 1 that the closing
                                 // relaxation of level l - 1 fills along with it (or null)
  float dt;         // step size of level 0 (1 for the GRU propagators, Sec. 3.3)
  hipStream_t s;
};

static PhiArgs phi_base(const FwdCtx& x, int l) {
  PhiArgs a;
  std::memset(&a, 0, sizeof(a));
  a.U = x.U;
  a.U3 = x.U3;
  a.b_h = x.b_h;
  a.P = x.P;
  a.u_in = x.ul[l];
  a.u = x.ul[l];
  a.g = x.gl[l];
  a.B = x.c->B;
  a.H = x.c->H;
  a.gamma = (float)x.lay->S[l] * x.dt;
  a.propagator = x.c->propagator;
  a.bf16 = kform(x.c->dtype);
  a.one_term = one_term(x.c->dtype);
  return a;
}

// F-relaxation (Alg. 1) or, with include_c, FC-relaxation on level l: sub-step j
// advances every interval from point i*cf+j-1 to i*cf+j.  All intervals move in one
// launch, so the C-sweep reads only values written by earlier launches (Jacobi in
// the coarse points).
// One level (the serial scan): whether the scan writes the adjoint coefficients along
// the way when asked to keep them.  With few rows per step the scan runs in the few-row
// kernels, where the five extra vectors per step cost more than one pass over all steps
// in the tile kernel afterwards; forward and backward calls decide by the same rule.
static bool serial_scan_keeps_coeffs(const mgrit_gru_cfg& c) { return c.B > 64; }

// Levels >= 1 whose coefficient vectors the forward call leaves (with MGRIT_KEEP_COEFFS and
// cf > 1) from the closing relaxation of the level above: level 1 always; deeper levels unless
// they are the coarsest one, whose few-row adjoint steps run faster on coefficients that the
// backward call has just written (0.4 us per step at 32 rows x 512) than the pass costs.
static bool forward_leaves_coeffs(int l, int L) { return l >= 1 && l < L && (l == 1 || l < L - 1); }

// zero_c: the coarse points 1.. of the level hold zero states (the caller's initial guess):
// the first sub-step reads nothing else outside the first interval.
// rhs_fused (may be null; F-sweeps of a level that has a coarser one): the sweep's first
// sub-step starts from the coarse points, the states the coarse level's operator is applied to
// in Eq. 11, and the contraction U h does not depend on the step size: that launch also
// evaluates the coarse step and leaves  R u' - Phi_c(R u')  in the coarse right-hand side
// array (mode STEP_RELAX_RHS).  *rhs_fused tells the caller whether such a launch ran.
// first_done: the first sub-step of the sweep is in place already (see vcycle_fwd).
static int relax_fwd(const FwdCtx& x, int l, bool include_c, bool f_points_current = false,
                     bool emit = false, bool zero_c = false, bool* rhs_fused = nullptr,
                     bool first_done = false) {
  const long long cf = x.c->cf, S = x.lay->S[l];
  const int nint = (int)(x.lay->N[l] / cf);
  if (rhs_fused) *rhs_fused = false;
  // f_points_current: the F-points already equal the propagation of their coarse
  // points (they were written by the closing F-relaxation of the previous cycle of
  // this call and nothing changed since), so recomputing them would reproduce the
  // same bits; only the C-sweep remains.
  for (long long j = f_points_current ? cf : (first_done ? 2 : 1); j < cf + (include_c ? 1 : 0);
       ++j) {
    PhiArgs a = phi_base(x, l);
    a.mode = STEP_RELAX;
    if (emit && x.emit_kap && l == 0) {
      // this sweep's values are final: the step from point o-1 to o is the one the
      // adjoint linearises, so its coefficient vectors are written along the way
      a.mode = STEP_RELAX_KAPPA;
      a.uc = x.emit_kap;
      a.kappa_width = 5 * x.c->H;
    }
    a.nk = nint;
    a.in = Idx{j - 1, cf};
    a.o = Idx{j, cf};
    a.p = Idx{j * S - 1, cf * S};
    if (emit && j == 1 && cf > 1 && x.emit_kapl[l + 1]) {
      // the first sub-step starts from the coarse points, whose values are final: they are the
      // states the steps of level l + 1 are linearised at, and the contraction U h is the same
      // for both step sizes, so this launch also leaves the coefficient vectors of level l + 1
      // (step from its point i to i + 1, row i + 1)
      a.mode = l == 0 ? STEP_RELAX_KAPPA2 : STEP_RELAX_CK;
      a.gc = x.emit_kapl[l + 1];
      a.a = Idx{1, 1};
      a.gamma2 = (float)x.lay->S[l + 1] * x.dt;
      a.dp2 = (cf * S - 1 - a.p.off) * x.c->B * 3LL * x.c->H;   // P row (i + 1) cf S - 1
    }
    if (zero_c && j == 1 && cf > 1) a.zero_from = x.c->B;   // rows of the intervals 1..
    if (rhs_fused && j == 1 && cf > 1 && !include_c && a.mode == STEP_RELAX &&
        !prop_is_lstm(x.c->propagator)) {
      // interval i: coarse step from coarse point i to i + 1 (level point (i + 1) cf)
      a.mode = STEP_RELAX_RHS;
      a.gc = x.gl[l + 1];
      a.a = Idx{1, 1};
      a.gamma2 = (float)x.lay->S[l + 1] * x.dt;
      const long long width = x.c->propagator == PROP_ODE_DEMO ? x.c->H : 3LL * x.c->H;
      a.dp2 = (cf * S - 1 - a.p.off) * x.c->B * width;       // P row (i + 1) cf S - 1
      a.do2 = (cf - a.o.off) * x.c->B * (long long)x.c->H;   // level point (i + 1) cf
      *rhs_fused = true;
    }
    const bool overlap = (cf == 1);   // reads and writes would share points
    if (overlap) a.u = x.tmp;
    CHECK_HIP(launch_phi_step(a, x.s));
    if (overlap)
      CHECK_HIP(launch_copy_points(x.ul[l], x.tmp, a.o, a.o, nint, (long long)a.B * a.H, x.s));
  }
  return MGRIT_OK;
}

// first_f_done (coarse levels): the iterate is the restricted one and the parent's residual
// launch has written the values of the first relaxation sub-step, R u' - R r, already.
static int vcycle_fwd(const FwdCtx& x, int l, bool f_points_current = false, bool last = false,
                      bool zero_guess = false, bool first_f_done = false) {
  const long long cf = x.c->cf, S = x.lay->S[l], N = x.lay->N[l];
  const int L = x.lay->L;
  if (l == L - 1) {
    // coarsest level: serial propagation (Appendix A.1)
    for (long long k = 1; k <= N; ++k) {
      PhiArgs a = phi_base(x, l);
      a.mode = STEP_RELAX;
      if (l == 0 && x.emit_kap) {        // one level: the serial scan itself
        a.mode = STEP_RELAX_KAPPA;
        a.uc = x.emit_kap;
        a.kappa_width = 5 * x.c->H;
      }
      a.nk = 1;
      a.in = Idx{k - 1, 0};
      a.o = Idx{k, 0};
      a.p = Idx{k * S - 1, 0};
      CHECK_HIP(launch_phi_step(a, x.s));
    }
    return MGRIT_OK;
  }
  int rc;
  // Alg. 2 line 1
  const bool cur = l == 0 && f_points_current;
  const bool zc = l == 0 && zero_guess && !cur;
  bool rhs_fused = false;
  if (l == 0 && x.c->fine_relax == 0) {
    if ((rc = relax_fwd(x, l, false, cur, false, zc, &rhs_fused))) return rc;
  } else {
    if ((rc = relax_fwd(x, l, true, cur, false, zc, nullptr, first_f_done))) return rc;
    if ((rc = relax_fwd(x, l, false, false, false, false, &rhs_fused))) return rc;
  }
  const int Nc = (int)(N / cf);
  const long long Sc = x.lay->S[l + 1];
  bool child_first_done = false;
  {  // lines 2-3: residual at the coarse points, restricted state
    PhiArgs a = phi_base(x, l);
    a.mode = STEP_RESID;
    a.nk = Nc;
    a.in = Idx{cf - 1, cf};
    a.o = Idx{cf, cf};
    a.p = Idx{cf * S - 1, cf * S};
    a.a = Idx{1, 1};
    a.uc = x.ul[l + 1];
    a.gc = x.gl[l + 1];
    a.norm = l == 0 ? x.norm : nullptr;
    a.resid_adds = rhs_fused ? 1 : 0;     // completes g_c = (R u' - Phi_c(R u')) - R r
    // A coarse level that relaxes starts with an F-sweep from the restricted iterate; its first
    // sub-step gives Phi_c(R u')_k + g_k = (R u')_k - (R r)_k at the points k = 1 (mod cf): this
    // launch writes them.  (Only with the fused right-hand side: a separate right-hand-side
    // launch reads the restricted iterate from the coarse array.)
    child_first_done = rhs_fused && cf > 1 && l + 1 < L - 1;
    if (child_first_done) {
      a.ff_cf = (int)cf;
      a.ff_rem = 1;
    }
    CHECK_HIP(launch_phi_step(a, x.s));
  }
  if (!rhs_fused) {  // line 4, right-hand side of Eq. 11: g_c = A_c(R u') - R r
    PhiArgs a = phi_base(x, l + 1);
    a.mode = STEP_RHS;
    a.nk = Nc;
    a.in = Idx{0, 1};
    a.o = Idx{1, 1};
    a.p = Idx{Sc - 1, Sc};
    CHECK_HIP(launch_phi_step(a, x.s));
  }
  if ((rc = vcycle_fwd(x, l + 1, false, last, false, child_first_done))) return rc;
  // line 5 at the coarse points: u'_{cf j} + (v_j - u'_{cf j}) = v_j.  F-points
  // would receive the same correction but are overwritten by line 6.
  CHECK_HIP(launch_copy_points(x.ul[l], x.ul[l + 1], Idx{cf, cf}, Idx{1, 1}, Nc,
                               (long long)x.c->B * x.c->H, x.s));
  // line 6
  return relax_fwd(x, l, false, false, last);
}

static int run_projection(const mgrit_gru_cfg* c, const Layout& lay, char* base, const void* W,
                          const float* b_i, const void* x, hipStream_t s) {
  if (c->flags & MGRIT_REUSE_PROJECTION) return MGRIT_OK;
  if (c->dtype == MGRIT_F32_BF16X3) {
    CHECK_HIP(launch_split3((const float*)W, base + lay.W3, 3LL * c->H * c->D, s));
    W = base + lay.W3;
  }
  // GRU: three gates; demonstration ODE: one block; LSTM: four gates of the hidden width c->H / 2
  const int width = c->propagator == PROP_ODE_DEMO ? c->H
                    : prop_is_lstm(c->propagator) ? 2 * c->H : 3 * c->H;
  CHECK_HIP(launch_projection(x, W, b_i, (float*)(base + lay.P), (long long)c->T * c->B, width,
                              c->D, kform(c->dtype), s));
  return MGRIT_OK;
}

// ode_dt != 0: the demonstration ODE (W = Bw[H,D], U = A[H,H], b_i = b, b_h unused) with
// level-0 step size ode_dt; the propagator field of the caller's cfg is not read.
// lstm: the LSTM step (W[4H,D], U[4H,H], b_i[4H], b_h[4H]; h0 and h are state pairs (h | c) of
// width 2H); cfg->propagator selects its implicit or explicit form.
static int forward_impl(const mgrit_gru_cfg* cin, bool serial, const void* W, const void* U,
                        const float* b_i, const float* b_h, const void* x, const float* h0,
                        float* h, float* resnorm, void* ws, size_t ws_bytes, void* stream,
                        float ode_dt = 0.f, bool lstm = false) {
  if (!cin) return MGRIT_E_NULL;
  mgrit_gru_cfg c = *cin;
  const bool ode = ode_dt != 0.f;
  if (ode) {
    if (!(ode_dt > 0.f) || !(ode_dt < 1e30f)) return MGRIT_E_SIZE;
    c.propagator = MGRIT_PROP_IMPLICIT;     // (any valid value for the checks below)
  }
  int rc = check_cfg(&c, !serial);
  if (rc) return rc;
  if ((ode || lstm) && (c.dtype != MGRIT_F32 || c.flags != 0)) return MGRIT_E_UNSUPPORTED;
  if (!W || !U || !b_i || !b_h || !x || !h0 || !h || !ws) return MGRIT_E_NULL;
  if (misaligned(W) || misaligned(U) || misaligned(x) || misaligned(h0) || misaligned(h) ||
      misaligned(ws))
    return MGRIT_E_ALIGN;
  if (ode) c.propagator = PROP_ODE_DEMO;
  if (lstm) {
    // the drivers move states of width 2H (h | c); the step kernels contract over the h half
    c.propagator = c.propagator == MGRIT_PROP_IMPLICIT ? PROP_LSTM_IMPLICIT : PROP_LSTM_CLASSIC;
    c.H *= 2;
  }
  if (serial) {
    c.levels = 1;
    c.cf = 1;
    c.iters = 1;
    c.fine_relax = 1;
  }
  Layout lay;
  make_layout(&c, &lay);
  if (ws_bytes < lay.total) return MGRIT_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)ws;
  const int pwidth = ode ? c.H : lstm ? 2 * c.H : 3 * c.H;
  WsRecord rec = ws_record_get(ws);
  if ((c.flags & MGRIT_REUSE_PROJECTION) && !proj_matches(rec, c, pwidth, x, W, b_i))
    return MGRIT_E_STATE;
  if ((c.flags & MGRIT_KEEP_COEFFS) && c.iters < 1) return MGRIT_E_SIZE;
  // from here on the workspace changes: note what it will hold when this call's work is done
  if (!(c.flags & MGRIT_REUSE_PROJECTION)) proj_note(rec, c, pwidth, x, W, b_i);
  rec.have_coeffs = (c.flags & MGRIT_KEEP_COEFFS) != 0;   // the states change: older vectors are stale
  rec.ccfg = c;
  rec.cserial = serial;
  rec.ch = h;
  ws_record_put(ws, rec);
  (void)hipGetLastError();   // an error left by earlier, unrelated work is not this call's

  FwdCtx ctx;
  ctx.c = &c;
  ctx.lay = &lay;
  ctx.U = U;
  ctx.U3 = nullptr;
  if (c.dtype == MGRIT_F32_BF16X3) {
    ctx.U3 = base + lay.U3;
    CHECK_HIP(launch_split3((const float*)U, base + lay.U3, 3LL * c.H * c.H, s));
  }
  ctx.b_h = b_h;
  ctx.P = (const float*)(base + lay.P);
  ctx.dt = ode ? ode_dt : 1.f;
  ctx.s = s;
  ctx.tmp = (float*)(base + lay.tmp);
  ctx.ul[0] = h;
  ctx.gl[0] = nullptr;
  for (int l = 1; l < lay.L; ++l) {
    ctx.ul[l] = (float*)(base + lay.u[l]);
    ctx.gl[l] = (float*)(base + lay.g[l]);
  }
  double* norm = (double*)(base + lay.norm);
  // MGRIT_KEEP_COEFFS: the closing F-relaxation of the last cycle (the serial scan, with
  // one level) also leaves the adjoint coefficient vectors of the steps it takes
  ctx.emit_kap = (c.flags & MGRIT_KEEP_COEFFS) ? (float*)(base + lay.kap[0]) : nullptr;
  if (lay.L == 1 && !serial_scan_keeps_coeffs(c)) ctx.emit_kap = nullptr;
  for (int l = 0; l < MAX_LEVELS; ++l)
    ctx.emit_kapl[l] = (ctx.emit_kap && forward_leaves_coeffs(l, lay.L))
                           ? (float*)(base + lay.kap[l]) : nullptr;

  if ((rc = run_projection(&c, lay, base, W, b_i, x, s))) return rc;
  const long long BH = (long long)c.B * c.H;
  for (int l = 0; l < lay.L; ++l)   // point 0 of every level is the initial condition
    CHECK_HIP(launch_copy_points(ctx.ul[l], h0, Idx{0, 0}, Idx{0, 0}, 1, BH, s));
  if (resnorm && c.iters > 0) CHECK_HIP(launch_fill_f64(norm, c.iters, 0.0, s));
  for (int it = 0; it < c.iters; ++it) {
    ctx.norm = resnorm ? norm + it : nullptr;
    const bool zero_guess = it == 0 && (c.flags & MGRIT_ZERO_STATE_GUESS) && !serial;
    if ((rc = vcycle_fwd(ctx, 0, it > 0, it == c.iters - 1, zero_guess))) return rc;
  }
  if (resnorm && !serial) CHECK_HIP(launch_sqrt_to_float(norm, resnorm, c.iters, s));
  return MGRIT_OK;
}

// ---------------------------------------------------------------------------
// adjoint drivers (time reversed: point N_l is fixed, steps run k -> k-1)
// ---------------------------------------------------------------------------
struct BwdCtx {
  const mgrit_gru_cfg* c;
  const Layout* lay;
  const void *UT, *UT3;
  const float* kap[MAX_LEVELS];
  float* wl[MAX_LEVELS];
  float* gl[MAX_LEVELS];
  float* tmp;
  double* norm;
  hipStream_t s;
};

static AdjArgs adj_base(const BwdCtx& x, int l) {
  AdjArgs a;
  std::memset(&a, 0, sizeof(a));
  a.UT = x.UT;
  a.UT3 = x.UT3;
  a.kap = x.kap[l];
  a.kw = (l == 0 ? 5 : 4) * x.c->H;
  a.w_in = x.wl[l];
  a.w = x.wl[l];
  a.g = x.gl[l];
  a.B = x.c->B;
  a.H = x.c->H;
  a.bf16 = kform(x.c->dtype);
  a.one_term = one_term(x.c->dtype);
  return a;
}

// Relaxation of the reversed recurrence: interval i hangs below coarse point
// (i+1)*cf; sub-step j moves from point (i+1)cf-j+1 to (i+1)cf-j with the
// coefficients of level step (i+1)cf-j+1.
//
// lo (a multiple of cf, or null): on entry the adjoint and the right-hand side of the
// level are known to be zero at every point below *lo.  The recurrence is linear and
// homogeneous, so an interval whose upper coarse point lies below *lo stays zero and is
// left out of the launches; on return *lo is the bound that holds after the sweep (one
// interval lower).
// first_done: the first sub-step of the sweep is in place already (see vcycle_bwd).
static int relax_bwd(const BwdCtx& x, int l, bool include_c, bool f_points_current = false,
                     long long* lo = nullptr, bool first_done = false) {
  const long long cf = x.c->cf;
  const int nint = (int)(x.lay->N[l] / cf);
  long long i0 = 0;                        // first interval that can hold non-zero values
  if (lo) {
    i0 = *lo / cf - 1;
    if (i0 < 0) i0 = 0;
    *lo = i0 * cf;
  }
  for (long long j = f_points_current ? cf : (first_done ? 2 : 1); j < cf + (include_c ? 1 : 0);
       ++j) {
    AdjArgs a = adj_base(x, l);
    a.mode = STEP_RELAX;
    a.nk = nint - (int)i0;
    a.in = Idx{cf - j + 1 + i0 * cf, cf};
    a.k = a.in;
    a.o = Idx{cf - j + i0 * cf, cf};
    const bool overlap = (cf == 1);
    if (overlap) a.w = x.tmp;
    CHECK_HIP(launch_adj_step(a, x.s));
    if (overlap)
      CHECK_HIP(launch_copy_points(x.wl[l], x.tmp, a.o, a.o, a.nk, (long long)a.B * a.H, x.s));
  }
  return MGRIT_OK;
}

// The adjoint recurrence is linear, so the coarse equation of Eq. 11 can be written for the
// error: with v = R w' + e its right-hand side A_c(R w') - R r turns into -R r and its initial
// guess R w' into zero; every relaxation and coarse solve then produces e where the scheme for
// v produces v - R w', and the correction adds e at the coarse points.  The iterates are those
// of Eq. 11 (up to rounding) without the launch that applies A_c to R w'.
//
// lo_in: bound below which the iterate and the right-hand side of this level are zero on entry
// (see relax_bwd; 0 = nothing known).
// first_f_done (coarse levels): the parent's residual launch has written the values of the
// first relaxation sub-step from the zero guess, -R r, already.
static int vcycle_bwd(const BwdCtx& x, int l, bool f_points_current = false,
                      long long lo_in = 0, bool first_f_done = false) {
  const long long cf = x.c->cf, N = x.lay->N[l];
  const int L = x.lay->L;
  if (l == L - 1) {
    for (long long k = N; k >= 1; --k) {
      AdjArgs a = adj_base(x, l);
      a.mode = STEP_RELAX;
      a.nk = 1;
      a.in = Idx{k, 0};
      a.k = Idx{k, 0};
      a.o = Idx{k - 1, 0};
      CHECK_HIP(launch_adj_step(a, x.s));
    }
    return MGRIT_OK;
  }
  int rc;
  const bool cur = l == 0 && f_points_current;
  long long lo = lo_in;
  long long* plo = lo > 0 && cf > 1 ? &lo : nullptr;
  if (!plo) lo = 0;
  if (l == 0 && x.c->fine_relax == 0) {
    if ((rc = relax_bwd(x, l, false, cur, plo))) return rc;
  } else {
    if ((rc = relax_bwd(x, l, true, cur, plo, first_f_done))) return rc;
    if ((rc = relax_bwd(x, l, false, false, plo))) return rc;
  }
  const int Nc = (int)(N / cf);
  // coarse points below lo have a zero iterate, a zero successor and a zero right-hand
  // side: their residual is zero and is written as such
  const long long iR = lo / cf;            // first coarse point with a non-zero residual
  // A coarse level that relaxes starts with an F-sweep from its zero guess; the first sub-step
  // gives g_k = -(R r)_k at the points k = cf - 1 (mod cf): the residual launch writes them
  // (not in a cycle that skips zero intervals).
  const bool child_first_done = cf > 1 && l + 1 < L - 1 && iR == 0;
  const long long BH = (long long)x.c->B * x.c->H;
  if (iR > 0) {
    CHECK_HIP(launch_zero_f32(x.wl[l + 1], iR * BH, x.s));
    CHECK_HIP(launch_zero_f32(x.gl[l + 1], iR * BH, x.s));
  }
  {  // residual at coarse points i*cf, i = iR..Nc-1; coarse right-hand side -R r, zero guess
    AdjArgs a = adj_base(x, l);
    a.mode = STEP_RESID;
    a.nk = Nc - (int)iR;
    a.in = Idx{1 + iR * cf, cf};
    a.k = a.in;
    a.o = Idx{iR * cf, cf};
    a.a = Idx{iR, 1};
    a.wc = x.wl[l + 1];
    a.gc = x.gl[l + 1];
    a.norm = l == 0 ? x.norm : nullptr;
    if (child_first_done) {
      a.ff_cf = (int)cf;
      a.ff_rem = (int)cf - 1;
    }
    CHECK_HIP(launch_adj_step(a, x.s));
  }
  // on the coarse level iterate and right-hand side are zero below iR
  if ((rc = vcycle_bwd(x, l + 1, false, iR / cf * cf, child_first_done))) return rc;
  // correction at the coarse points: w'_{cf i} + e_i (the coarse solve carries e below iR too)
  CHECK_HIP(launch_add_points(x.wl[l], x.wl[l + 1], Idx{0, cf}, Idx{0, 1}, Nc, BH, x.s));
  return relax_bwd(x, l, false);
}

static int backward_impl(const mgrit_gru_cfg* cin, bool serial, const void* W, const void* U,
                         const float* b_i, const float* b_h, const void* x, const float* h,
                         const float* dL_dhT, const float* dL_dh, float* w, float* resnorm,
                         float* dW, float* dU, float* db_i, float* db_h, float* dx, void* ws,
                         size_t ws_bytes, void* stream) {
  int rc = check_cfg(cin, !serial);
  if (rc) return rc;
  // a loss on every state: dL_dh[(T+1),B,H] is the source term of the adjoint
  // recurrence, i.e. the right-hand side of the level-0 equation; its last row is
  // the terminal condition
  if (dL_dh) dL_dhT = dL_dh + (size_t)cin->T * cin->B * cin->H;
  if (!W || !U || !b_i || !b_h || !x || !h || !dL_dhT || !w || !ws) return MGRIT_E_NULL;
  if (misaligned(dL_dh) || misaligned(dx)) return MGRIT_E_ALIGN;
  const int ngrad = (dW != nullptr) + (dU != nullptr) + (db_i != nullptr) + (db_h != nullptr);
  if (ngrad != 0 && ngrad != 4) return MGRIT_E_NULL;
  if (serial && ngrad != 4) return MGRIT_E_NULL;
  if (misaligned(W) || misaligned(U) || misaligned(x) || misaligned(h) || misaligned(dL_dhT) ||
      misaligned(w) || misaligned(ws) || misaligned(dW) || misaligned(dU))
    return MGRIT_E_ALIGN;
  mgrit_gru_cfg c = *cin;
  if (serial) {
    c.levels = 1;
    c.cf = 1;
    c.iters = 1;
    c.fine_relax = 1;
  }
  Layout lay;
  make_layout(&c, &lay);
  if (ws_bytes < lay.total) return MGRIT_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* base = (char*)ws;
  const float* P = (const float*)(base + lay.P);
  const long long BH = (long long)c.B * c.H;
  WsRecord rec = ws_record_get(ws);
  if ((c.flags & MGRIT_REUSE_PROJECTION) && !proj_matches(rec, c, 3 * c.H, x, W, b_i))
    return MGRIT_E_STATE;
  if ((c.flags & MGRIT_REUSE_COEFFS) && !coeffs_match(rec, c, serial, h)) return MGRIT_E_STATE;
  if (!(c.flags & MGRIT_REUSE_PROJECTION)) proj_note(rec, c, 3 * c.H, x, W, b_i);
  // this call completes (or rebuilds) the vectors of every step for these states: they stay
  // valid for a later backward call on the same problem
  rec.have_coeffs = true;
  rec.ccfg = c;
  rec.cserial = serial;
  rec.ch = h;
  ws_record_put(ws, rec);
  (void)hipGetLastError();   // an error left by earlier, unrelated work is not this call's

  if ((rc = run_projection(&c, lay, base, W, b_i, x, s))) return rc;
  const int bf16 = kform(c.dtype) == 1;
  CHECK_HIP(launch_transpose(U, base + lay.UT, 3 * c.H, c.H, bf16, s));
  if (c.dtype == MGRIT_F32_BF16X3) {
    CHECK_HIP(launch_split3((const float*)U, base + lay.U3, 3LL * c.H * c.H, s));
    CHECK_HIP(launch_split3((const float*)(base + lay.UT), base + lay.UT3, 3LL * c.H * c.H, s));
  }

  BwdCtx ctx;
  ctx.c = &c;
  ctx.lay = &lay;
  ctx.UT = base + lay.UT;
  ctx.UT3 = base + lay.UT3;
  ctx.s = s;
  ctx.tmp = (float*)(base + lay.tmp);
  ctx.wl[0] = w;
  ctx.gl[0] = const_cast<float*>(dL_dh);   // level 0 only reads its right-hand side
  for (int l = 0; l < lay.L; ++l) {
    ctx.kap[l] = (const float*)(base + lay.kap[l]);
    if (l > 0) {
      ctx.wl[l] = (float*)(base + lay.u[l]);
      ctx.gl[l] = (float*)(base + lay.g[l]);
    }
    // coefficient vectors of every step of level l: step k is linearised at the
    // forward state of level point k-1 (fine point (k-1)*S) and input x_{k*S}
    PhiArgs a;
    std::memset(&a, 0, sizeof(a));
    a.U = U;
    a.U3 = base + lay.U3;
    a.bf16 = kform(c.dtype);
    a.one_term = one_term(c.dtype);
    a.b_h = b_h;
    a.P = P;
    a.u_in = h;
    a.uc = (float*)(base + lay.kap[l]);
    a.kappa_width = (l == 0 ? 5 : 4) * c.H;
    a.B = c.B;
    a.H = c.H;
    a.gamma = (float)lay.S[l];
    a.propagator = c.propagator;
    a.mode = STEP_KAPPA;
    a.nk = (int)lay.N[l];
    a.in = Idx{0, lay.S[l]};
    a.p = Idx{lay.S[l] - 1, lay.S[l]};
    a.o = Idx{1, 1};
    if (l == 0 && (c.flags & MGRIT_REUSE_COEFFS)) {
      // the forward call left the coefficients of every step that ends in an F-point (all
      // steps, with one level): only the steps into the coarse points i*cf remain
      if (lay.L == 1) {
        if (serial_scan_keeps_coeffs(c)) a.nk = 0;   // else: the scan left none, full pass
      } else {
        a.nk = (int)(lay.N[0] / c.cf);
        a.in = Idx{c.cf - 1, c.cf};
        a.p = Idx{c.cf - 1, c.cf};
        a.o = Idx{c.cf, c.cf};
      }
    }
    // ... and, from the coarse points the first sub-step of every level's closing relaxation
    // starts at, the coefficients of every step of the next level
    if ((c.flags & MGRIT_REUSE_COEFFS) && c.cf > 1 && forward_leaves_coeffs(l, lay.L)) a.nk = 0;
    CHECK_HIP(launch_phi_step(a, s));
    // the terminal condition w_T = dL/dh_T is the fixed end point of level 0; the coarse levels
    // solve for errors, whose end point is zero
    if (l == 0)
      CHECK_HIP(launch_copy_points(ctx.wl[l], dL_dhT, Idx{lay.N[l], 0}, Idx{0, 0}, 1, BH, s));
    else
      CHECK_HIP(launch_zero_f32(ctx.wl[l] + lay.N[l] * BH, BH, s));
  }
  double* norm = (double*)(base + lay.norm);
  if (resnorm && c.iters > 0) CHECK_HIP(launch_fill_f64(norm, c.iters, 0.0, s));
  for (int it = 0; it < c.iters; ++it) {
    ctx.norm = resnorm ? norm + it : nullptr;
    // the caller's zero initial guess with a terminal loss term: everything below point T
    // is zero when the first cycle starts
    // (with a loss term on every state the flag also declares rows 0..T-1 of that term zero)
    const bool zero_guess = it == 0 && (c.flags & MGRIT_ZERO_ADJOINT_GUESS) && !serial;
    if ((rc = vcycle_bwd(ctx, 0, it > 0, zero_guess ? lay.N[0] : 0))) return rc;
  }
  if (resnorm && !serial) CHECK_HIP(launch_sqrt_to_float(norm, resnorm, c.iters, s));
  if (ngrad == 4)
    CHECK_HIP(launch_param_grads(ctx.kap[0], w, h, x, dW, dU, db_i, db_h,
                                 (float*)(base + lay.part), c.T, c.B, c.D, c.H, kform(c.dtype),
                                 one_term(c.dtype), s));
  if (dx) {
    CHECK_HIP(launch_transpose(W, base + lay.WT, 3 * c.H, c.D, bf16, s));
    const void* WT = base + lay.WT;
    if (c.dtype == MGRIT_F32_BF16X3) {
      CHECK_HIP(launch_split3((const float*)WT, base + lay.W3, 3LL * c.H * c.D, s));
      WT = base + lay.W3;
    }
    CHECK_HIP(launch_input_grads(ctx.kap[0], w, WT, dx, c.T, c.B, c.D, c.H, kform(c.dtype),
                                 one_term(c.dtype), s));
  }
  return MGRIT_OK;
}

}  // namespace mg

// ---------------------------------------------------------------------------
// exported symbols
// ---------------------------------------------------------------------------
using namespace mg;

extern "C" {

int mgrit_gru_workspace_bytes(const mgrit_gru_cfg* cfg, size_t* bytes) {
  if (!bytes) return MGRIT_E_NULL;
  int rc = check_cfg(cfg, true);
  if (rc) return rc;
  Layout lay;
  make_layout(cfg, &lay);
  *bytes = lay.total;
  return MGRIT_OK;
}

int gru_serial_scan(const mgrit_gru_cfg* cfg, const void* W, const void* U, const float* b_i,
                    const float* b_h, const void* x, const float* h0, float* h_out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(cfg, true, W, U, b_i, b_h, x, h0, h_out, nullptr, workspace,
                      workspace_bytes, stream);
}

int mgrit_gru_forward(const mgrit_gru_cfg* cfg, const void* W, const void* U, const float* b_i,
                      const float* b_h, const void* x, const float* h0, float* h_inout,
                      float* resnorm_out, void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(cfg, false, W, U, b_i, b_h, x, h0, h_inout, resnorm_out, workspace,
                      workspace_bytes, stream);
}

int mgrit_gru_forward_static(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                             const float* b_i, const float* b_h, const void* x, const float* h0,
                             float* h_inout, float* resnorm_out, void* stream) {
  // everything that can be refused is refused before the device is touched
  int rc = check_cfg(cfg, true);
  if (rc) return rc;
  if (cfg->flags & ~MGRIT_ZERO_STATE_GUESS) return MGRIT_E_UNSUPPORTED;
  Layout lay;
  make_layout(cfg, &lay);
  if (lay.total > (size_t)MGRIT_STATIC_SCRATCH_BYTES) return MGRIT_E_WORKSPACE;
  if (!W || !U || !b_i || !b_h || !x || !h0 || !h_inout) return MGRIT_E_NULL;
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  t_no_prof = true;       // event objects are runtime allocations: none in this call
  rc = forward_impl(cfg, false, W, U, b_i, b_h, x, h0, h_inout, resnorm_out, ws,
                    (size_t)MGRIT_STATIC_SCRATCH_BYTES, stream);
  t_no_prof = false;
  return rc;
}

int mgrit_lstm_workspace_bytes(const mgrit_gru_cfg* cfg, size_t* bytes) {
  if (!bytes) return MGRIT_E_NULL;
  int rc = check_cfg(cfg, true);
  if (rc) return rc;
  mgrit_gru_cfg c = *cfg;
  c.H *= 2;                    // state pairs (h | c)
  Layout lay;
  make_layout(&c, &lay);
  *bytes = lay.total;
  return MGRIT_OK;
}

int lstm_serial_scan(const mgrit_gru_cfg* cfg, const float* W, const float* U, const float* b_i,
                     const float* b_h, const float* x, const float* u0, float* u_out,
                     void* workspace, size_t workspace_bytes, void* stream) {
  return forward_impl(cfg, true, W, U, b_i, b_h, x, u0, u_out, nullptr, workspace,
                      workspace_bytes, stream, 0.f, true);
}

int mgrit_lstm_forward(const mgrit_gru_cfg* cfg, const float* W, const float* U,
                       const float* b_i, const float* b_h, const float* x, const float* u0,
                       float* u_inout, float* resnorm_out, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return forward_impl(cfg, false, W, U, b_i, b_h, x, u0, u_inout, resnorm_out, workspace,
                      workspace_bytes, stream, 0.f, true);
}

int ode_serial_scan(const mgrit_gru_cfg* cfg, float dt, const float* A, const float* Bw,
                    const float* b, const float* d, const float* h0, float* h_out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!(dt > 0.f)) return MGRIT_E_SIZE;
  return forward_impl(cfg, true, Bw, A, b, b, d, h0, h_out, nullptr, workspace, workspace_bytes,
                      stream, dt);
}

int mgrit_ode_forward(const mgrit_gru_cfg* cfg, float dt, const float* A, const float* Bw,
                      const float* b, const float* d, const float* h0, float* h_inout,
                      float* resnorm_out, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (!(dt > 0.f)) return MGRIT_E_SIZE;
  return forward_impl(cfg, false, Bw, A, b, b, d, h0, h_inout, resnorm_out, workspace,
                      workspace_bytes, stream, dt);
}

int gru_serial_scan_backward(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                             const float* b_i, const float* b_h, const void* x, const float* h,
                             const float* dL_dhT, float* w_out, float* dW, float* dU, float* db_i,
                             float* db_h, void* workspace, size_t workspace_bytes, void* stream) {
  return backward_impl(cfg, true, W, U, b_i, b_h, x, h, dL_dhT, nullptr, w_out, nullptr, dW, dU,
                       db_i, db_h, nullptr, workspace, workspace_bytes, stream);
}

int gru_serial_scan_backward_steps(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                                   const float* b_i, const float* b_h, const void* x,
                                   const float* h, const float* dL_dh, float* w_out, float* dW,
                                   float* dU, float* db_i, float* db_h, float* dx,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (!dL_dh) return MGRIT_E_NULL;
  return backward_impl(cfg, true, W, U, b_i, b_h, x, h, nullptr, dL_dh, w_out, nullptr, dW, dU,
                       db_i, db_h, dx, workspace, workspace_bytes, stream);
}

int mgrit_gru_backward_steps(const mgrit_gru_cfg* cfg, const void* W, const void* U,
                             const float* b_i, const float* b_h, const void* x, const float* h,
                             const float* dL_dh, float* w_inout, float* resnorm_out, float* dW,
                             float* dU, float* db_i, float* db_h, float* dx, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!dL_dh) return MGRIT_E_NULL;
  return backward_impl(cfg, false, W, U, b_i, b_h, x, h, nullptr, dL_dh, w_inout, resnorm_out, dW,
                       dU, db_i, db_h, dx, workspace, workspace_bytes, stream);
}

int mgrit_gru_backward(const mgrit_gru_cfg* cfg, const void* W, const void* U, const float* b_i,
                       const float* b_h, const void* x, const float* h, const float* dL_dhT,
                       float* w_inout, float* resnorm_out, float* dW, float* dU, float* db_i,
                       float* db_h, void* workspace, size_t workspace_bytes, void* stream) {
  return backward_impl(cfg, false, W, U, b_i, b_h, x, h, dL_dhT, nullptr, w_inout, resnorm_out,
                       dW, dU, db_i, db_h, nullptr, workspace, workspace_bytes, stream);
}

const char* mgrit_gru_strerror(int code) {
  switch (code) {
    case MGRIT_OK: return "ok";
    case MGRIT_E_NULL: return "null pointer";
    case MGRIT_E_SIZE: return "size out of range";
    case MGRIT_E_HIERARCHY: return "cf^(levels-1) does not divide T";
    case MGRIT_E_ENUM: return "unknown enum or flag value";
    case MGRIT_E_WORKSPACE: return "workspace too small";
    case MGRIT_E_ALIGN: return "width not a multiple of 4 (8 unless dtype is MGRIT_F32) or pointer not 16-byte aligned";
    case MGRIT_E_LAUNCH: return "HIP launch failed";
    case MGRIT_E_UNSUPPORTED: return "unsupported configuration";
    case MGRIT_E_STATE:
      return "workspace does not hold what MGRIT_REUSE_PROJECTION / MGRIT_REUSE_COEFFS asks for";
    default: return "unknown error";
  }
}

int mgrit_gru_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  const bool was = g_prof;
  g_prof = on != 0;
  if (g_prof && !was) {
    // switching on starts a fresh record (events of unread launches are released, not waited
    // for); switching off keeps the record for the reads that follow
    for (auto& r : g_recs) {
      (void)hipEventDestroy(r.e0);
      (void)hipEventDestroy(r.e1);
    }
    g_recs.clear();
  }
  return MGRIT_OK;
}

int mgrit_gru_profile_read(int kind, int64_t* launches, double* ms, double* flops, double* bytes) {
  return mgrit_gru_profile_read_shape(kind, -1, -1, launches, ms, flops, bytes);
}

int mgrit_gru_profile_read_shape(int kind, int64_t rows, int mode, int64_t* launches, double* ms,
                                 double* flops, double* bytes) {
  if (!launches || !ms || !flops || !bytes) return MGRIT_E_NULL;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  *launches = 0;
  *ms = *flops = *bytes = 0.0;
  std::vector<ProfRec> keep;
  for (auto& r : g_recs) {
    if (r.kind != kind || (rows >= 0 && r.rows != rows) || (mode >= 0 && r.mode != mode)) {
      keep.push_back(r);
      continue;
    }
    float t = 0.f;
    if (hipEventSynchronize(r.e1) == hipSuccess && hipEventElapsedTime(&t, r.e0, r.e1) == hipSuccess) {
      *launches += 1;
      *ms += t;
      *flops += r.flops;
      *bytes += r.bytes;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  g_recs.swap(keep);
  return MGRIT_OK;
}

}  // extern "C"
