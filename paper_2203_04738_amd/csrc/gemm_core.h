// Workgroup-tile fp32 MFMA contraction core for gfx950 (CDNA4), shared by the
// projection GEMM, the fused GRU step and its adjoint.
//
// C[TM x (NG*TN)] += A[TM x K] * B[(NG*TN) x K]^T with both operands
// K-contiguous in memory ("NT" form).  The tile is staged through LDS in
// K-slices of TK = 32 floats and consumed by v_mfma_f32_32x32x2_f32:
//   - operand A: lane l supplies A[i = l%32][k = l/32]
//   - operand B: lane l supplies B[k = l/32][j = l%32]
//   - result:    register v of lane l holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l%32]
// A lane reads four consecutive k (one ds_read_b128) and feeds four MFMAs; the
// two half-waves take k-offsets 0..3 and 4..7 of every group of eight, so A and
// B agree on which k each MFMA contracts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mg {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int TK = 32;        // K-slice staged per iteration
constexpr int LDS_PAD = 4;    // floats; keeps rows 16-byte aligned and spreads banks
constexpr int LDS_LD = TK + LDS_PAD;

template <int WM_, int WN_, int BM_, int BN_, int NG_>
struct TileCfg {
  static constexpr int WM = WM_, WN = WN_, BM = BM_, BN = BN_, NG = NG_;
  static constexpr int NWAVES = WM * WN;
  static constexpr int NT = NWAVES * 64;
  static constexpr int TM = WM * BM * 32;
  static constexpr int TN = WN * BN * 32;       // per gate group
  static constexpr int BROWS = NG * TN;
  static constexpr int A_CHUNKS = (TM * (TK / 4) + NT - 1) / NT;     // float4 per thread
  static constexpr int B_CHUNKS = (BROWS * (TK / 4) + NT - 1) / NT;
  static constexpr int LDS_FLOATS = (TM + BROWS) * LDS_LD;
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

// One pass over K.  LoadA(s, row_in_tile, k) and LoadB(s, row_in_tile, k) return
// the float4 at columns k..k+3 of that tile row (zeros outside the matrix); k is a
// multiple of 4 and s is the index of the calling thread's chunk (its tile row is
// fixed for the whole pass, so callers can keep one base pointer per chunk:
// chunk s of thread tid covers tile row (tid + s*NT)/8).
template <class C, class LoadA, class LoadB>
__device__ inline void gemm_nt_tile(Acc<C>& acc, int K, LoadA loadA, LoadB loadB, float* lds) {
  float* As = lds;
  float* Bs = lds + C::TM * LDS_LD;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / C::WN;
  const int wn = wave % C::WN;
  const int li = lane & 31;
  const int lh = lane >> 5;

  floatx4 ra[C::A_CHUNKS];
  floatx4 rb[C::B_CHUNKS];

  auto fetch = [&](int k0) {
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      int q = tid + s * C::NT;
      int row = q / (TK / 4), c4 = q % (TK / 4);
      if (C::TM * (TK / 4) % C::NT == 0 || row < C::TM) ra[s] = loadA(s, row, k0 + c4 * 4);
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      int q = tid + s * C::NT;
      int row = q / (TK / 4), c4 = q % (TK / 4);
      if (C::BROWS * (TK / 4) % C::NT == 0 || row < C::BROWS) rb[s] = loadB(s, row, k0 + c4 * 4);
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int s = 0; s < C::A_CHUNKS; ++s) {
      int q = tid + s * C::NT;
      int row = q / (TK / 4), c4 = q % (TK / 4);
      if (C::TM * (TK / 4) % C::NT == 0 || row < C::TM)
        *reinterpret_cast<floatx4*>(&As[row * LDS_LD + c4 * 4]) = ra[s];
    }
#pragma unroll
    for (int s = 0; s < C::B_CHUNKS; ++s) {
      int q = tid + s * C::NT;
      int row = q / (TK / 4), c4 = q % (TK / 4);
      if (C::BROWS * (TK / 4) % C::NT == 0 || row < C::BROWS)
        *reinterpret_cast<floatx4*>(&Bs[row * LDS_LD + c4 * 4]) = rb[s];
    }
  };

  const int nkt = (K + TK - 1) / TK;
  fetch(0);
  stash();
  __syncthreads();
  for (int kt = 0; kt < nkt; ++kt) {
    if (kt + 1 < nkt) fetch((kt + 1) * TK);
#pragma unroll
    for (int c = 0; c < TK / 8; ++c) {
      floatx4 a4[C::BM];
#pragma unroll
      for (int a = 0; a < C::BM; ++a)
        a4[a] = *reinterpret_cast<const floatx4*>(
            &As[((wm * C::BM + a) * 32 + li) * LDS_LD + c * 8 + lh * 4]);
#pragma unroll
      for (int g = 0; g < C::NG; ++g)
#pragma unroll
        for (int b = 0; b < C::BN; ++b) {
          floatx4 b4 = *reinterpret_cast<const floatx4*>(
              &Bs[(g * C::TN + (wn * C::BN + b) * 32 + li) * LDS_LD + c * 8 + lh * 4]);
#pragma unroll
          for (int a = 0; a < C::BM; ++a) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc.v[g][a][b] =
                  __builtin_amdgcn_mfma_f32_32x32x2f32(a4[a][e], b4[e], acc.v[g][a][b], 0, 0, 0);
          }
        }
    }
    __syncthreads();
    if (kt + 1 < nkt) {
      stash();
      __syncthreads();
    }
  }
}

// Coordinates of accumulator element e of block (a, b) of this wave inside the
// workgroup tile.
template <class C>
__device__ inline void acc_coord(int a, int b, int e, int& row, int& col) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave / C::WN, wn = wave % C::WN;
  row = (wm * C::BM + a) * 32 + 8 * (e / 4) + 4 * (lane >> 5) + (e & 3);
  col = (wn * C::BN + b) * 32 + (lane & 31);
}

__device__ inline floatx4 ldg4(const float* p) { return *reinterpret_cast<const floatx4*>(p); }
__device__ inline floatx4 zero4() {
  floatx4 z = {0.f, 0.f, 0.f, 0.f};
  return z;
}

}  // namespace mg
