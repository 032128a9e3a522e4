// Workgroup-level float64 tile GEMM on the gfx950 matrix cores.
//
// One workgroup of 256 threads (4 wavefronts arranged 2 x 2) produces a
// (32*TM) x (32*TN) tile of  sum_k A(i,k) * B(k,j)  with v_mfma_f64_16x16x4.
// Operands are fetched element-wise through functors, staged in LDS in a
// [k][i] / [k][j] layout, and consumed as 16x4 / 4x16 fragments:
//   A fragment: lane l holds A(i = l % 16, k = l / 16)
//   B fragment: lane l holds B(k = l / 16, j = l % 16)
//   D fragment: lane l, register r holds D(i = 4*r + l / 16, j = l % 16)
// (the D layout of the f64 instruction differs from the f32 ones; it was
// confirmed on hardware).  At 64 cycles per instruction the matrix pipe needs
// two doubles per lane per instruction, so plain 8-byte LDS reads keep it busy.
#pragma once
#include "common.h"

namespace ptq {

constexpr int kGemmBK = 16;

template <int TM, int TN>
struct DgemmTile {
  static constexpr int BM = 32 * TM;
  static constexpr int BN = 32 * TN;
  static constexpr int PA = BM + 16;  // LDS pitches (doubles)
  static constexpr int PB = BN + 16;
  static constexpr int kSmemDoubles = kGemmBK * (PA + PB);
  static constexpr int EA = BM * kGemmBK / 256;  // elements per thread per k-tile
  static constexpr int EB = BN * kGemmBK / 256;
};

// fa(i, k): element of A for tile-local row i < rows and absolute k in [kbeg, kend).
// fb(k, j): element of B for absolute k and tile-local column j < cols.
// The functors are only ever called with indices inside those ranges (out-of-range
// tile positions are clamped to (0, kbeg) and the value discarded), so they must be
// plain loads without branches: every load of a k-tile is then in flight at once.
// A_KFAST / B_KFAST say which index is contiguous in memory so that the
// thread -> element map coalesces.
template <int TM, int TN, bool A_KFAST, bool B_KFAST, class FA, class FB>
__device__ __forceinline__ void dgemm_mainloop(f64x4 (&acc)[TM][TN], FA fa, FB fb, int rows, int cols,
                                               int kbeg, int kend, double* smem) {
  using T = DgemmTile<TM, TN>;
  double* sa = smem;
  double* sb = smem + kGemmBK * T::PA;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  double ra[T::EA], rb[T::EB];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int p = 0; p < T::EA; ++p) {
      const int e = tid + 256 * p;
      const int i = A_KFAST ? e / kGemmBK : e % T::BM;
      const int k = A_KFAST ? e % kGemmBK : e / T::BM;
      const bool ok = (k0 + k < kend) & (i < rows);
      const double v = fa(ok ? i : 0, ok ? k0 + k : kbeg);
      ra[p] = ok ? v : 0.0;
    }
#pragma unroll
    for (int p = 0; p < T::EB; ++p) {
      const int e = tid + 256 * p;
      const int j = B_KFAST ? e / kGemmBK : e % T::BN;
      const int k = B_KFAST ? e % kGemmBK : e / T::BN;
      const bool ok = (k0 + k < kend) & (j < cols);
      const double v = fb(ok ? k0 + k : kbeg, ok ? j : 0);
      rb[p] = ok ? v : 0.0;
    }
  };
  auto stash = [&]() {
#pragma unroll
    for (int p = 0; p < T::EA; ++p) {
      const int e = tid + 256 * p;
      const int i = A_KFAST ? e / kGemmBK : e % T::BM;
      const int k = A_KFAST ? e % kGemmBK : e / T::BM;
      sa[k * T::PA + i] = ra[p];
    }
#pragma unroll
    for (int p = 0; p < T::EB; ++p) {
      const int e = tid + 256 * p;
      const int j = B_KFAST ? e / kGemmBK : e % T::BN;
      const int k = B_KFAST ? e % kGemmBK : e / T::BN;
      sb[k * T::PB + j] = rb[p];
    }
  };

  if (kbeg >= kend) return;
  fetch(kbeg);
  for (int k0 = kbeg; k0 < kend; k0 += kGemmBK) {
    __syncthreads();  // previous tile fully consumed
    stash();
    __syncthreads();
    if (k0 + kGemmBK < kend) fetch(k0 + kGemmBK);
#pragma unroll
    for (int kk = 0; kk < kGemmBK; kk += 4) {
      double a[TM], b[TN];
      const int kr = kk + (lane >> 4);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) a[tm] = sa[kr * T::PA + wm * 16 * TM + tm * 16 + (lane & 15)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) b[tn] = sb[kr * T::PB + wn * 16 * TN + tn * 16 + (lane & 15)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[tm], b[tn], acc[tm][tn], 0, 0, 0);
    }
  }
}

// Visit every accumulator element with its tile-local (i, j).
template <int TM, int TN, class FC>
__device__ __forceinline__ void dgemm_foreach(const f64x4 (&acc)[TM][TN], FC fc) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = wm * 16 * TM + tm * 16 + 4 * r + (lane >> 4);
        const int j = wn * 16 * TN + tn * 16 + (lane & 15);
        fc(i, j, acc[tm][tn][r]);
      }
}

template <int TM, int TN>
__device__ __forceinline__ void dgemm_zero(f64x4 (&acc)[TM][TN]) {
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) acc[tm][tn] = f64x4{0.0, 0.0, 0.0, 0.0};
}

}  // namespace ptq
