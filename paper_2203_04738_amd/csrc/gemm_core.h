// Workgroup-tile fp32 MFMA contraction core for gfx950 (CDNA4), shared by the
// projection GEMM, the fused GRU step and its adjoint.
//
// C[TM x (NG*TN)] += A[TM x K] * B[(NG*TN) x K]^T with both operands
// K-contiguous in memory ("NT" form).  The tile is staged through LDS in
// K-slices of TK floats and consumed by v_mfma_f32_32x32x2_f32:
//   - operand A: lane l supplies A[i = l%32][k = l/32]
//   - operand B: lane l supplies B[k = l/32][j = l%32]
//   - result:    register v of lane l holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32]
// A lane reads four consecutive k (one ds_read_b128) and feeds four MFMAs; the
// two half-waves take k-offsets 0..3 and 4..7 of every group of eight, so A and
// B agree on which k each MFMA contracts.
//
// Pipeline: the global loads of slice kt+1 are issued into registers before the
// MFMAs of slice kt; with NBUF = 2 they are written to the other LDS buffer
// after the MFMAs and one barrier per slice suffices.  Inside a slice the LDS
// fragments of k-group c+1 are read while the MFMAs of group c issue.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ inline floatx4 ldg4(const float* p) { return *reinterpret_cast<const floatx4*>(p); }
// streamed operand (read once per launch): loaded with the non-temporal hint so that
// it does not displace the weights and state rows the tiles share in L2
__device__ inline floatx4 ldg4_stream(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const floatx4*>(p));
}
__device__ inline floatx4 zero4() {
  floatx4 z = {0.f, 0.f, 0.f, 0.f};
  return z;
}
struct Identity4 {
  __device__ inline floatx4 operator()(const floatx4& v) const { return v; }
};

constexpr int LDS_PAD = 4;    // floats; keeps rows 16-byte aligned and spreads banks

// KS > 1: K-split inside the workgroup for launches with few rows.  KS groups of
// WM*WN waves all compute the same output tile, group ks contracting the k-groups
// [ks*NC/KS, (ks+1)*NC/KS) of every staged slice (TK is KS times longer, the loads
// stay coalesced); the partial sums are added in the epilogue staging.
template <int WM_, int WN_, int BM_, int BN_, int NG_, int TK_ = 32, int NBUF_ = 1, int KS_ = 1>
struct TileCfg {
  static constexpr int WM = WM_, WN = WN_, BM = BM_, BN = BN_, NG = NG_, TK = TK_, NBUF = NBUF_;
  static constexpr int KS = KS_;
  static constexpr int MINWG = 2;               // resident workgroups per CU planned for
  static constexpr int NWAVES = WM * WN * KS;
  static constexpr int NT = NWAVES * 64;
  static constexpr int TM = WM * BM * 32;
  static constexpr int TN = WN * BN * 32;       // per gate group
  static constexpr int BROWS = NG * TN;
  static constexpr int LD = TK + LDS_PAD;       // LDS row stride in floats
  static constexpr int CPR = TK / 4;            // float4 chunks per tile row
  static constexpr int A_CHUNKS = (TM * CPR) / NT;     // float4 per thread
  static constexpr int B_CHUNKS = (BROWS * CPR) / NT;
  static constexpr int BUF_FLOATS = (TM + BROWS) * LD;
  static constexpr int LDS_FLOATS = NBUF * BUF_FLOATS;
  static_assert((TM * CPR) % NT == 0 && (BROWS * CPR) % NT == 0, "tile rows must divide evenly");
  static_assert(TK % (8 * KS) == 0, "TK must be a multiple of 8 per K-split group");
};

// Accumulators of one wave: acc[g][bm][bn] is a 32x32 block.
template <class C>
struct Acc {
  floatx16 v[C::NG][C::BM][C::BN];
  __device__ inline void zero() {
#pragma unroll
    for (int g = 0; g < C::NG; ++g)
#pragma unroll
      for (int a = 0; a < C::BM; ++a)
#pragma unroll
        for (int b = 0; b < C::BN; ++b)
#pragma unroll
          for (int e = 0; e < 16; ++e) v[g][a][b][e] = 0.f;
  }
};

// Tile row covered by chunk s of this thread (fixed for the whole pass).
template <class C>
__device__ inline int chunk_row(int s) { return (threadIdx.x + s * C::NT) / C::CPR; }

// One pass over K.
//   loadA(s, k) / loadB(s, k): raw global load(s) for the calling thread's chunk s
//     at columns k..k+3 of its tile row (k a multiple of 4, always < K: the core
//     clamps it).  The returned value (any trivially copyable type) stays in
//     registers while the MFMAs of the current slice run.
//   finA(raw) / finB(raw): turn the raw value into the float4 that goes to LDS;
//     they run after the MFMAs, so nothing waits on the loads before that.
// KTAIL: K is not a multiple of TK; columns >= K are zero-filled.
template <class C, bool KTAIL, class LoadA, class LoadB, class FinA, class FinB>
__device__ inline void gemm_nt_tile(Acc<C>& acc, int K, LoadA loadA, LoadB loadB, FinA finA,
                                    FinB finB, float* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = (tid >> 6) % (C::WM * C::WN);
  const int ks = (tid >> 6) / (C::WM * C::WN);      // K-split group of this wave
  const int wm = wave / C::WN;
  const int wn = wave % C::WN;
  const int li = lane & 31;
  const int lh = lane >> 5;
  constexpr int NC = C::TK / 8 / C::KS;  // k-groups of eight per slice and K-split group
  constexpr int NB = C::NG * C::BN;      // B fragments per k-group

  decltype(loadA(0, 0)) ra[C::A_CHUNKS];
  decltype(loadB(0, 0)) rb[C::B_CHUNKS];

  auto fetch = [&](int k0) {
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      int k = k0 + ((tid + s * C::NT) % C::CPR) * 4;
      if (KTAIL && k >= K) k = K - 4;
      ra[s] = loadA(s, k);
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      int k = k0 + ((tid + s * C::NT) % C::CPR) * 4;
      if (KTAIL && k >= K) k = K - 4;
      rb[s] = loadB(s, k);
    }
  };
  auto stash = [&](float* buf, int k0) {
    float* As = buf;
    float* Bs = buf + C::TM * C::LD;
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      const int q = tid + s * C::NT;
      floatx4 v = finA(ra[s]);
      if (KTAIL && k0 + (q % C::CPR) * 4 >= K) v = zero4();
      *reinterpret_cast<floatx4*>(&As[(q / C::CPR) * C::LD + (q % C::CPR) * 4]) = v;
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      const int q = tid + s * C::NT;
      floatx4 v = finB(rb[s]);
      if (KTAIL && k0 + (q % C::CPR) * 4 >= K) v = zero4();
      *reinterpret_cast<floatx4*>(&Bs[(q / C::CPR) * C::LD + (q % C::CPR) * 4]) = v;
    }
  };
  // fragment addresses of this lane inside a buffer (first k-group of its K-split group)
  const int a_off = ((wm * C::BM) * 32 + li) * C::LD + lh * 4 + ks * NC * 8;
  const int b_off = C::TM * C::LD + ((wn * C::BN) * 32 + li) * C::LD + lh * 4 + ks * NC * 8;
  auto read_frags = [&](const float* buf, int c, floatx4 (&fa)[C::BM], floatx4 (&fb)[NB]) {
#pragma unroll
    for (int a = 0; a < C::BM; ++a)
      fa[a] = *reinterpret_cast<const floatx4*>(&buf[a_off + a * 32 * C::LD + c * 8]);
#pragma unroll
    for (int g = 0; g < C::NG; ++g)
#pragma unroll
      for (int b = 0; b < C::BN; ++b)
        fb[g * C::BN + b] = *reinterpret_cast<const floatx4*>(
            &buf[b_off + (g * C::TN + b * 32) * C::LD + c * 8]);
  };
  auto mma = [&](const floatx4 (&fa)[C::BM], const floatx4 (&fb)[NB]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int g = 0; g < C::NG; ++g)
#pragma unroll
        for (int b = 0; b < C::BN; ++b)
#pragma unroll
          for (int a = 0; a < C::BM; ++a)
            acc.v[g][a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                fa[a][e], fb[g * C::BN + b][e], acc.v[g][a][b], 0, 0, 0);
  };

  const int nkt = (K + C::TK - 1) / C::TK;
  fetch(0);
  stash(lds, 0);
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    const float* cur = lds + (C::NBUF == 2 ? (kt & 1) * C::BUF_FLOATS : 0);
    float* nxt = lds + (C::NBUF == 2 ? ((kt + 1) & 1) * C::BUF_FLOATS : 0);
    const bool more = kt + 1 < nkt;
    if (more) fetch((kt + 1) * C::TK);
    // the loads above stay in flight across the MFMAs; their consumers are below
    __builtin_amdgcn_sched_barrier(0);
    floatx4 fa[2][C::BM];
    floatx4 fb[2][NB];
    // waves that are feeding the MFMA pipe go first at instruction issue: waves of the
    // other resident workgroup that are staging or in their epilogue fill the gaps
    __builtin_amdgcn_s_setprio(2);
    read_frags(cur, 0, fa[0], fb[0]);
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (c + 1 < NC) read_frags(cur, c + 1, fa[(c + 1) & 1], fb[(c + 1) & 1]);
      mma(fa[c & 1], fb[c & 1]);
      if (c + 1 < NC) {
        // issue order inside this k-group: one LDS read of the next group's fragments,
        // then a share of this group's MFMAs, and so on (left to itself the scheduler
        // sinks the reads next to their first use)
        constexpr int NR = C::BM + NB;
        constexpr int MPR = (4 * C::BM * NB) / NR;
#pragma unroll
        for (int i = 0; i < NR; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // one DS read
          __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);   // MPR MFMAs
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(0);
    if (C::NBUF == 2) {
      if (more) stash(nxt, (kt + 1) * C::TK);
      __syncthreads();
    } else {
      __syncthreads();
      if (more) {
        stash(nxt, (kt + 1) * C::TK);
        __syncthreads();
      }
    }
  }
}

// XCD-aware tile order.  Workgroups are dispatched round-robin over the 8 XCDs
// (workgroup id % 8), each with its own L2.  Row tile rt is pinned to XCD rt % 8
// and, inside an XCD, consecutive workgroups walk the column tiles of one row
// tile, so the A rows of a row tile are fetched into one L2 only and the
// workgroups resident on an XCD share a small set of A tiles.
// The 1-D grid has 8 * ncol * ceil(nrow / 8) workgroups; returns false for the
// padding ones.
constexpr int NXCD = 8;
__host__ __device__ inline long long xcd_grid(long long nrow, int ncol) {
  return ((nrow + NXCD - 1) / NXCD) * NXCD * ncol;
}
__device__ inline bool xcd_tile(long long bid, long long nrow, int ncol, long long& rt, int& ct) {
  const int xcd = (int)(bid % NXCD);
  const long long j = bid / NXCD;
  ct = (int)(j % ncol);
  rt = (j / ncol) * NXCD + xcd;
  return rt < nrow;
}

// Coordinates of accumulator element e of block (a, b) of this wave inside the
// workgroup tile.
template <class C>
__device__ inline void acc_coord(int a, int b, int e, int& row, int& col) {
  const int lane = threadIdx.x & 63;
  const int wave = (threadIdx.x >> 6) % (C::WM * C::WN);
  const int wm = wave / C::WN, wn = wave % C::WN;
  row = (wm * C::BM + a) * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e & 3);
  col = (wn * C::BN + b) * 32 + (lane & 31);
}

// Staging of the accumulators for the epilogue.  The MFMA result layout gives a lane
// one column and sixteen scattered rows, which would make every global access of the
// epilogue a 4-byte one; the sums are therefore passed through LDS, one 32-row block
// row of every wave per pass, and picked up again with a thread owning four
// consecutive columns of a row ("item"), so that epilogue operands and outputs move
// as 16-byte accesses covering whole row segments.
template <class C>
struct EpiStage {
  static constexpr int ROWS = C::WM * 32;              // tile rows staged per pass
  static constexpr int LD = C::TN + 8;                 // 4*LD = 32 (mod 64): conflict-free writes
  static constexpr int C4 = C::TN / 4;                 // float4 columns of a tile row
  static constexpr int NITEM = ROWS * C4;              // items of a pass
  static constexpr int ITEMS = (NITEM + C::NT - 1) / C::NT;   // items per thread and pass
  static constexpr int RSTEP = C::NT / C4;             // staged rows between items of a thread
  static constexpr int SLAB = C::NG * ROWS * LD;       // floats of one K-split group
  static constexpr int FLOATS = C::KS * SLAB;
  static_assert(C::NT % C4 == 0, "threads must cover whole staged rows");
  static_assert(NITEM % C::NT == 0 || C::NT % NITEM == 0, "epilogue items must divide evenly");

  // block row ba of every wave -> stage[ks][g][row][col]
  __device__ static inline void write(const Acc<C>& acc, int ba, float* stage) {
    const int lane = threadIdx.x & 63;
    const int wave = (threadIdx.x >> 6) % (C::WM * C::WN);
    const int ks = (threadIdx.x >> 6) / (C::WM * C::WN);
    const int wm = wave / C::WN, wn = wave % C::WN;
    const int li = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int g = 0; g < C::NG; ++g)
#pragma unroll
      for (int bb = 0; bb < C::BN; ++bb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = wm * 32 + 8 * (e / 4) + 4 * lh + (e & 3);
          const int col = (wn * C::BN + bb) * 32 + li;
          stage[ks * SLAB + (g * ROWS + row) * LD + col] = acc.v[g][ba][bb][e];
        }
  }
  // threads beyond the items of a pass (workgroups wider than the staged block) idle
  __device__ static inline bool active() { return C::NT <= NITEM || (int)threadIdx.x < NITEM; }
  __device__ static inline int col4() { return threadIdx.x % C4; }
  __device__ static inline int staged_row(int it) {
    const int rp = threadIdx.x / C4 + it * RSTEP;
    return rp < ROWS ? rp : ROWS - 1;
  }
  // row of the workgroup tile behind staged row rp of pass ba
  __device__ static inline int tile_row(int rp, int ba) {
    return ((rp / 32) * C::BM + ba) * 32 + (rp & 31);
  }
  // sum over the K-split groups of gate g at (rp, c4)
  __device__ static inline floatx4 read(const float* stage, int g, int rp, int c4) {
    floatx4 v = *reinterpret_cast<const floatx4*>(&stage[(g * ROWS + rp) * LD + c4 * 4]);
#pragma unroll
    for (int k = 1; k < C::KS; ++k)
      v += *reinterpret_cast<const floatx4*>(&stage[k * SLAB + (g * ROWS + rp) * LD + c4 * 4]);
    return v;
  }
};

}  // namespace mg
