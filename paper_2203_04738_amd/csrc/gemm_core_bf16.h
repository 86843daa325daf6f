// Workgroup-tile bf16 MFMA contraction core for gfx950 (CDNA4): the same "NT"
// tile product as gemm_core.h, consumed by v_mfma_f32_32x32x16_bf16 with fp32
// accumulation, for the variant whose inputs and weights are stored in bf16.
//
// Operand B (weights) is bf16 in memory.  Operand A is either bf16 in memory
// (the input sequence x) or fp32 (hidden states, adjoint values).  An fp32 operand
// is rounded to bf16 on its way to LDS (one tile, one MFMA per block: the usual
// mixed-precision contraction), or, in the two-term form, written as TWO bf16 tiles,
// hi = bf16(a) and lo = bf16(a - hi), with two MFMAs per block, hi*B + lo*B: that keeps
// 16 mantissa bits of the fp32 state in the product, so the only rounding the method
// sees beyond fp32 is the one already present in the stored bf16 weights.
//
// With NP = 3 both operands are fp32 VALUES carried as three bf16 terms each
// (a = a0 + a1 + a2 exactly: 3 x 8 mantissa bits); the contraction keeps the six
// products a_t * b_u with t + u <= 2 and drops the three of relative size 2^-24 and
// below, so the fp32 accumulators receive what an fp32 product would have given them,
// at the rate of the bf16 matrix pipe.  A is split on its way to LDS, B arrives already
// split (three arrays, prepared once per call).
//
// A lane supplies eight consecutive k of its row (one ds_read_b128) per MFMA, the
// two half-waves taking k-offsets 0..7 and 8..15 of each group of sixteen; A and B
// use the same assignment, so the contraction is independent of how the
// instruction numbers k inside a lane.
#pragma once
#include <type_traits>

#include "gemm_core.h"

namespace mg {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short bf16_t;     // storage type of bf16 arrays at the ABI

struct F32x8 {
  floatx4 lo4, hi4;                // columns k..k+3 and k+4..k+7
};

__device__ inline bf16x8 ldg8h(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

struct Bf16x8x3 {
  bf16x8 p[3];                     // the three terms of eight consecutive values
};
__device__ inline const bf16x8& operand_term(const bf16x8& v, int) { return v; }
__device__ inline const bf16x8& operand_term(const Bf16x8x3& v, int u) { return v.p[u]; }

__device__ inline void split_bf16_3(const F32x8& v, bf16x8& t0, bf16x8& t1, bf16x8& t2) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float a = i < 4 ? v.lo4[i] : v.hi4[i - 4];
    const __bf16 h = (__bf16)a;
    const float r1 = a - (float)h;           // exact
    const __bf16 m = (__bf16)r1;
    t0[i] = h;
    t1[i] = m;
    t2[i] = (__bf16)(r1 - (float)m);         // the difference is exact
  }
}

__device__ inline void split_bf16(const F32x8& v, bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    hi[i] = (__bf16)v.lo4[i];
    hi[4 + i] = (__bf16)v.hi4[i];
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    lo[i] = (__bf16)(v.lo4[i] - (float)hi[i]);
    lo[4 + i] = (__bf16)(v.hi4[i] - (float)hi[4 + i]);
  }
}

// DEPTH: K-slices whose global loads are in flight at once (each in its own set of
// registers).  The MFMAs of a bf16 slice take a quarter of the time of an fp32 one, less
// than the latency of the loads for the next slice; with DEPTH = 3 a slice's loads have
// three slice times to arrive.  MINWG: resident workgroups per CU the register budget
// is planned for.
// NP: 1 = operands as stored (A optionally in two terms), 3 = three terms per operand.
// TKB: elements per K-slice and K-split group.
// A2: an fp32 operand A goes to the MFMAs as two bf16 terms (hi + lo); false: as one, rounded
// to nearest (what mixed-precision training feeds its matrix pipe).
template <int WM_, int WN_, int BM_, int BN_, int NG_, bool SPLIT_A_, int KS_ = 1, int DEPTH_ = 1,
          int MINWG_ = 2, int NP_ = 1, int TKB_ = 64, bool A2_ = true>
struct TileCfgB {
  static constexpr int WM = WM_, WN = WN_, BM = BM_, BN = BN_, NG = NG_;
  static constexpr bool SPLIT_A = SPLIT_A_;
  static constexpr int DEPTH = DEPTH_, MINWG = MINWG_;
  static constexpr int KS = KS_;                // K-split groups of waves (see TileCfg)
  static constexpr int NP = NP_;
  static constexpr int TK = TKB_ * KS;          // bf16 elements per K-slice
  static constexpr int NA = NP == 3 ? 3 : (SPLIT_A && A2_) ? 2 : 1;   // A tiles in LDS
  static constexpr int NBP = NP == 3 ? 3 : 1;                // B tiles in LDS
  static constexpr int NTERM = NA > NBP ? NA : NBP;          // products kept: t + u < NTERM
  static constexpr int NWAVES = WM * WN * KS;
  static constexpr int NT = NWAVES * 64;
  static constexpr int TM = WM * BM * 32;
  static constexpr int TN = WN * BN * 32;
  static constexpr int BROWS = NG * TN;
  // LDS rows: padded by 16 bytes (an odd multiple of 16 bytes per row), or, for the three-term
  // tiles with 64-byte rows, unpadded with the four 16-byte chunks of a row exchanged by
  // bits 2-3 of the row number, so that sixteen neighbouring lanes cover all banks once both
  // when a slice is written (four rows x four chunks) and when it is read (sixteen rows).
  static constexpr bool SWZ = NP_ == 3 && KS_ == 1 && TKB_ == 32;
  static constexpr int LD = SWZ ? TK : TK + 8;  // LDS row stride in elements
  static constexpr int CPR = TK / 8;            // 16-byte chunks per tile row
  static constexpr int A_CHUNKS = (TM * CPR) / NT;
  static constexpr int B_CHUNKS = (BROWS * CPR) / NT;
  static constexpr int LDS_ELEMS = (NA * TM + NBP * BROWS) * LD;
  static_assert(SPLIT_A || NP == 1, "three-term operands are fp32 in memory");
  static_assert((TM * CPR) % NT == 0 && (BROWS * CPR) % NT == 0, "tile rows must divide evenly");
};

template <class C>
__device__ inline int chunk_row_b(int s) { return (threadIdx.x + s * C::NT) / C::CPR; }
// position of 16-byte chunk `chunk` inside LDS row `row`
template <class C>
__device__ inline int swz_chunk(int row, int chunk) {
  return C::SWZ ? chunk ^ ((row >> 2) & 3) : chunk;
}

// One pass over K (elements; a multiple of 8).
//   loadA(s, k): raw global load(s) for columns k..k+7 of the tile row of chunk s;
//   finA(raw): -> bf16x8 (SPLIT_A false) or F32x8 (SPLIT_A true), applied when the
//              slice is written to LDS;
//   loadB(s, k): -> bf16x8, or Bf16x8x3 (NP = 3).
template <class C, bool KTAIL, class LoadA, class LoadB, class FinA>
__device__ inline void gemm_nt_tile_bf16(Acc<C>& acc, int K, LoadA loadA, LoadB loadB, FinA finA,
                                         bf16_t* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = (tid >> 6) % (C::WM * C::WN);
  const int ks = (tid >> 6) / (C::WM * C::WN);      // K-split group of this wave
  const int wm = wave / C::WN;
  const int wn = wave % C::WN;
  const int li = lane & 31;
  const int lh = lane >> 5;
  constexpr int NC = C::TK / 16 / C::KS;            // k-groups of sixteen per slice and group
  constexpr int NB = C::NG * C::BN;
  constexpr int NFA = C::NA * C::BM;
  constexpr int NFB = C::NBP * NB;

  constexpr int DP = C::DEPTH;
  // register set d holds the raw loads of the slices kt = d (mod DP); every index into
  // these arrays is a constant once the loops below are unrolled
  decltype(loadA(0, 0)) ra[DP][C::A_CHUNKS];
  decltype(loadB(0, 0)) rb[DP][C::B_CHUNKS];

  auto fetch = [&](int d, int k0) {
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      int k = k0 + ((tid + s * C::NT) % C::CPR) * 8;
      if (KTAIL && k >= K) k = K - 8;
      ra[d][s] = loadA(s, k);
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      int k = k0 + ((tid + s * C::NT) % C::CPR) * 8;
      if (KTAIL && k >= K) k = K - 8;
      rb[d][s] = loadB(s, k);
    }
  };
  bf16_t* As = lds;                               // hi (or only) A tile, then lo tile
  bf16_t* Bs = lds + C::NA * C::TM * C::LD;
  auto stash = [&](int d, int k0) {
    bf16x8 z;
#pragma unroll
    for (int i = 0; i < 8; ++i) z[i] = (__bf16)0.f;
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      const int q = tid + s * C::NT;
      const int off = (q / C::CPR) * C::LD + swz_chunk<C>(q / C::CPR, q % C::CPR) * 8;
      const bool dead = KTAIL && k0 + (q % C::CPR) * 8 >= K;
      if constexpr (C::NA == 3) {
        bf16x8 t0, t1, t2;
        split_bf16_3(finA(ra[d][s]), t0, t1, t2);
        *reinterpret_cast<bf16x8*>(&As[off]) = dead ? z : t0;
        *reinterpret_cast<bf16x8*>(&As[C::TM * C::LD + off]) = dead ? z : t1;
        *reinterpret_cast<bf16x8*>(&As[2 * C::TM * C::LD + off]) = dead ? z : t2;
      } else if constexpr (C::SPLIT_A) {
        bf16x8 hi, lo;
        split_bf16(finA(ra[d][s]), hi, lo);
        *reinterpret_cast<bf16x8*>(&As[off]) = dead ? z : hi;
        if constexpr (C::NA == 2)
          *reinterpret_cast<bf16x8*>(&As[C::TM * C::LD + off]) = dead ? z : lo;
      } else {
        *reinterpret_cast<bf16x8*>(&As[off]) = dead ? z : finA(ra[d][s]);
      }
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      const int q = tid + s * C::NT;
      const bool dead = KTAIL && k0 + (q % C::CPR) * 8 >= K;
#pragma unroll
      for (int u = 0; u < C::NBP; ++u)
        *reinterpret_cast<bf16x8*>(
            &Bs[(u * C::BROWS + q / C::CPR) * C::LD + swz_chunk<C>(q / C::CPR, q % C::CPR) * 8]) =
            dead ? z : operand_term(rb[d][s], u);
    }
  };
  const int a_off = ((wm * C::BM) * 32 + li) * C::LD + lh * 8 + ks * NC * 16;
  const int b_off = ((wn * C::BN) * 32 + li) * C::LD + lh * 8 + ks * NC * 16;
  auto read_frags = [&](int c, bf16x8 (&fa)[NFA], bf16x8 (&fb)[NFB]) {
#pragma unroll
    for (int t = 0; t < C::NA; ++t)
#pragma unroll
      for (int a = 0; a < C::BM; ++a)
        fa[t * C::BM + a] = *reinterpret_cast<const bf16x8*>(
            &As[t * C::TM * C::LD + a_off + a * 32 * C::LD + c * 16]);
#pragma unroll
    for (int u = 0; u < C::NBP; ++u)
#pragma unroll
      for (int g = 0; g < C::NG; ++g)
#pragma unroll
        for (int b = 0; b < C::BN; ++b)
          fb[u * NB + g * C::BN + b] = *reinterpret_cast<const bf16x8*>(
              &Bs[u * C::BROWS * C::LD + b_off + (g * C::TN + b * 32) * C::LD + c * 16]);
  };
  auto mma = [&](const bf16x8 (&fa)[NFA], const bf16x8 (&fb)[NFB]) {
#pragma unroll
    for (int t = 0; t < C::NA; ++t)
#pragma unroll
      for (int u = 0; u < C::NBP; ++u) {
        if (t + u >= C::NTERM) continue;
#pragma unroll
        for (int g = 0; g < C::NG; ++g)
#pragma unroll
          for (int b = 0; b < C::BN; ++b)
#pragma unroll
            for (int a = 0; a < C::BM; ++a)
              acc.v[g][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                  fa[t * C::BM + a], fb[u * NB + g * C::BN + b], acc.v[g][a][b], 0, 0, 0);
      }
  };

  const int nkt = (K + C::TK - 1) / C::TK;
#pragma unroll
  for (int d = 0; d < DP; ++d)
    if (d < nkt) fetch(d, d * C::TK);
  stash(0, 0);
  __syncthreads();
  for (int kt0 = 0; kt0 < nkt; kt0 += DP) {
#pragma unroll
    for (int d = 0; d < DP; ++d) {
      const int kt = kt0 + d;
      if (kt < nkt) {
        // slice kt sits in LDS, so its register set is free for slice kt + DP
        if (kt + DP < nkt) fetch(d, (kt + DP) * C::TK);
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 fa[2][NFA];
        bf16x8 fb[2][NFB];
        __builtin_amdgcn_s_setprio(2);        // see gemm_core.h
        if constexpr (C::NP == 3) {
          // Three-term operands: the products of a k-group are issued in three units, one
          // per B term u (A terms 0..2-u against it: 18, 12 and 6 MFMAs for a 2 x 3 block
          // tile), and every fragment is requested one unit before its first use, a read
          // in front of each of the unit's first MFMAs.  B terms alternate between two
          // register sets; of the A terms only term 0 (used by every unit) needs two.
          bf16x8 a0[2][C::BM], a1[C::BM], a2[C::BM], bt[2][NB];
          // element offset of this lane's chunk of k-group c inside its rows (all rows a
          // lane reads are 32 apart: one exchange pattern, bits 2-3 of li)
          const int a_row = ((wm * C::BM) * 32 + li) * C::LD;
          const int b_row = ((wn * C::BN) * 32 + li) * C::LD;
          auto kpos = [&](int c) { return swz_chunk<C>(li, ks * NC * 2 + 2 * c + lh) * 8; };
          auto rdA = [&](int c, int t, bf16x8 (&f)[C::BM]) {
#pragma unroll
            for (int a = 0; a < C::BM; ++a)
              f[a] = *reinterpret_cast<const bf16x8*>(
                  &As[t * C::TM * C::LD + a_row + a * 32 * C::LD + kpos(c)]);
          };
          auto rdB = [&](int c, int u, bf16x8 (&f)[NB]) {
#pragma unroll
            for (int g = 0; g < C::NG; ++g)
#pragma unroll
              for (int b = 0; b < C::BN; ++b)
                f[g * C::BN + b] = *reinterpret_cast<const bf16x8*>(
                    &Bs[u * C::BROWS * C::LD + b_row + (g * C::TN + b * 32) * C::LD + kpos(c)]);
          };
          auto mm = [&](const bf16x8 (&f)[C::BM], const bf16x8 (&h)[NB]) {
#pragma unroll
            for (int g = 0; g < C::NG; ++g)
#pragma unroll
              for (int b = 0; b < C::BN; ++b)
#pragma unroll
                for (int a = 0; a < C::BM; ++a)
                  acc.v[g][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                      f[a], h[g * C::BN + b], acc.v[g][a][b], 0, 0, 0);
          };
          constexpr int UM = C::BM * NB;            // MFMAs of one (A term, B term) pair
          rdA(0, 0, a0[0]);
          rdB(0, 0, bt[0]);
          rdA(0, 2, a2);
          rdA(0, 1, a1);
          auto group = [&](auto more_tag, int c) {
            constexpr bool more = decltype(more_tag)::value;   // a k-group follows in this slice
            const int s0 = (3 * c) & 1;            // register set of B term 0 of this group
            // unit 0
            rdB(c, 1, bt[s0 ^ 1]);
            mm(a0[c & 1], bt[s0]);
            mm(a2, bt[s0]);
            mm(a1, bt[s0]);
#pragma unroll
            for (int i = 0; i < NB; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 3 * UM - NB, 0);
            __builtin_amdgcn_sched_barrier(0);
            // unit 1
            rdB(c, 2, bt[s0]);
            if constexpr (more) {
              rdA(c + 1, 2, a2);
              rdA(c + 1, 0, a0[(c + 1) & 1]);
            }
            mm(a0[c & 1], bt[s0 ^ 1]);
            mm(a1, bt[s0 ^ 1]);
            {
              constexpr int nr = NB + (more ? 2 * C::BM : 0);
              constexpr int np = nr < 2 * UM ? nr : 2 * UM;
#pragma unroll
              for (int i = 0; i < np; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
              }
              if constexpr (nr > np) __builtin_amdgcn_sched_group_barrier(0x100, nr - np, 0);
              if constexpr (2 * UM > np) __builtin_amdgcn_sched_group_barrier(0x008, 2 * UM - np, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            // unit 2
            if constexpr (more) {
              rdB(c + 1, 0, bt[s0 ^ 1]);
              rdA(c + 1, 1, a1);
            }
            mm(a0[c & 1], bt[s0]);
            if constexpr (more) {
              constexpr int nr = NB + C::BM;
              constexpr int np = nr < UM ? nr : UM;
#pragma unroll
              for (int i = 0; i < np; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
              }
              if constexpr (nr > np) __builtin_amdgcn_sched_group_barrier(0x100, nr - np, 0);
              if constexpr (UM > np) __builtin_amdgcn_sched_group_barrier(0x008, UM - np, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
          };
#pragma unroll
          for (int c = 0; c + 1 < NC; ++c) group(std::true_type(), c);
          group(std::false_type(), NC - 1);
        } else {
        read_frags(0, fa[0], fb[0]);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          if (c + 1 < NC) read_frags(c + 1, fa[(c + 1) & 1], fb[(c + 1) & 1]);
          mma(fa[c & 1], fb[c & 1]);
          if (c + 1 < NC) {
            // one LDS read of the next k-group, then a share of this group's MFMAs, in turn
            constexpr int NR = NFA + NB;
            constexpr int NM = C::NA * C::BM * NB;
            constexpr int MPR = NM / NR > 0 ? NM / NR : 1;
#pragma unroll
            for (int i = 0; i < NR; ++i) {
              __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
        __syncthreads();
        if (kt + 1 < nkt) {
          stash((d + 1) % DP, (kt + 1) * C::TK);
          __syncthreads();
        }
      }
    }
  }
}

// Element loads for the vector-FMA kernels: four consecutive weights as floats.
__device__ inline floatx4 ldg4w(const float* p) { return ldg4(p); }
__device__ inline floatx4 ldg4w(const bf16_t* p) {
  const uint2 r = *reinterpret_cast<const uint2*>(p);
  floatx4 v;
  v[0] = __uint_as_float(r.x << 16);
  v[1] = __uint_as_float(r.x & 0xffff0000u);
  v[2] = __uint_as_float(r.y << 16);
  v[3] = __uint_as_float(r.y & 0xffff0000u);
  return v;
}

}  // namespace mg
