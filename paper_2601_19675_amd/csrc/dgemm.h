// Workgroup-level float64 tile GEMM on the gfx950 matrix cores.
//
// One workgroup of 256 threads (4 wavefronts arranged 2 x 2) produces a
// (32*TM) x (32*TN) tile of  sum_k A(i,k) * B(k,j)  with v_mfma_f64_16x16x4.
// Operands are strided views of float64 matrices, staged in LDS in a
// [k][i] / [k][j] layout, and consumed as 16x4 / 4x16 fragments:
//   A fragment: lane l holds A(i = l % 16, k = l / 16)
//   B fragment: lane l holds B(k = l / 16, j = l % 16)
//   D fragment: lane l, register r holds D(i = 4*r + l / 16, j = l % 16)
// (the D layout of the f64 instruction differs from the f32 ones; it was
// confirmed on hardware).  At 64 cycles per instruction the matrix pipe needs
// two doubles per lane per instruction, so plain 8-byte LDS reads keep it busy;
// what has to be kept small is everything else a wave issues, because a wave
// issues in order and with one wave per SIMD nothing else fills the gaps.
// Hence: per-thread element offsets are computed once and advanced by one add
// per k-tile, loads for tile t+2 are issued before the MFMAs of tile t, and
// LDS is double-buffered so that there is one barrier per k-tile.
#pragma once
#include "common.h"

namespace ptq {

constexpr int kGemmBK = 16;

template <int TM, int TN>
struct DgemmTile {
  static constexpr int BM = 32 * TM;
  static constexpr int BN = 32 * TN;
  // LDS pitches (doubles): +2 spreads both the k-strided stores of a k-contiguous
  // operand and the four k-rows of a fragment read over all banks
  static constexpr int PA = BM + 2;
  static constexpr int PB = BN + 2;
  static constexpr int kStageDoubles = kGemmBK * (PA + PB);
  static constexpr int kSmemDoubles = 2 * kStageDoubles;
  static constexpr int EA = BM * kGemmBK / 256;  // elements per thread per k-tile
  static constexpr int EB = BN * kGemmBK / 256;
};

// element(o, k) = p[o * so + k * sk], o = row of A / column of B inside the tile.
// All offsets of one tile fit in 31 bits.
struct DView {
  const double* p;
  int so, sk;
};

struct DgemmIdentity {
  __device__ __forceinline__ double operator()(double v, int, int) const { return v; }
};

// fa(v, i, k) / fb(v, k, j) may transform a loaded value (tile-local i / j,
// absolute k); they run one k-tile after the load, just before the LDS store.
// `rows` x `cols` is the valid part of the tile, k runs over [kbeg, kend).
// KFAST says whether k is the contiguous index of the view (coalescing).
template <int TM, int TN, bool A_KFAST, bool B_KFAST, class FA, class FB>
__device__ __forceinline__ void dgemm_mainloop(f64x4 (&acc)[TM][TN], DView A, FA fa, DView B, FB fb, int rows,
                                               int cols, int kbeg, int kend, double* smem) {
  using T = DgemmTile<TM, TN>;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  if (kbeg >= kend) return;

  // fixed per-thread element coordinates and running offsets (at k-tile 0)
  int offa[T::EA], offb[T::EB];
  unsigned oka = 0, okb = 0;
#pragma unroll
  for (int p = 0; p < T::EA; ++p) {
    const int e = tid + 256 * p;
    const int i = A_KFAST ? e / kGemmBK : e % T::BM;
    const int k = A_KFAST ? e % kGemmBK : e / T::BM;
    oka |= (i < rows ? 1u : 0u) << p;
    offa[p] = (i < rows ? i : rows - 1) * A.so + (kbeg + k) * A.sk;
  }
#pragma unroll
  for (int p = 0; p < T::EB; ++p) {
    const int e = tid + 256 * p;
    const int j = B_KFAST ? e / kGemmBK : e % T::BN;
    const int k = B_KFAST ? e % kGemmBK : e / T::BN;
    okb |= (j < cols ? 1u : 0u) << p;
    offb[p] = (j < cols ? j : cols - 1) * B.so + (kbeg + k) * B.sk;
  }
  const int stepa = kGemmBK * A.sk, stepb = kGemmBK * B.sk;

  double ra[T::EA], rb[T::EB];
  // loads of the k-tile starting at k0 (its offsets are the current ones); only
  // the last tile can stick out of [kbeg, kend): there the k index is clamped
  auto fetch = [&](int k0) {
    if (k0 + kGemmBK <= kend) {
#pragma unroll
      for (int p = 0; p < T::EA; ++p) ra[p] = A.p[offa[p]];
#pragma unroll
      for (int p = 0; p < T::EB; ++p) rb[p] = B.p[offb[p]];
    } else {
#pragma unroll
      for (int p = 0; p < T::EA; ++p) {
        const int k = A_KFAST ? (tid + 256 * p) % kGemmBK : (tid + 256 * p) / T::BM;
        const int over = k0 + k - (kend - 1);
        ra[p] = A.p[offa[p] - (over > 0 ? over : 0) * A.sk];
      }
#pragma unroll
      for (int p = 0; p < T::EB; ++p) {
        const int k = B_KFAST ? (tid + 256 * p) % kGemmBK : (tid + 256 * p) / T::BN;
        const int over = k0 + k - (kend - 1);
        rb[p] = B.p[offb[p] - (over > 0 ? over : 0) * B.sk];
      }
    }
#pragma unroll
    for (int p = 0; p < T::EA; ++p) offa[p] += stepa;
#pragma unroll
    for (int p = 0; p < T::EB; ++p) offb[p] += stepb;
  };
  auto stash = [&](int k0, double* st) {
    double* sa = st;
    double* sb = st + kGemmBK * T::PA;
#pragma unroll
    for (int p = 0; p < T::EA; ++p) {
      const int e = tid + 256 * p;
      const int i = A_KFAST ? e / kGemmBK : e % T::BM;
      const int k = A_KFAST ? e % kGemmBK : e / T::BM;
      const bool ok = ((oka >> p) & 1u) && (k0 + k < kend);
      const double v = fa(ra[p], i, k0 + k);
      sa[k * T::PA + i] = ok ? v : 0.0;
    }
#pragma unroll
    for (int p = 0; p < T::EB; ++p) {
      const int e = tid + 256 * p;
      const int j = B_KFAST ? e / kGemmBK : e % T::BN;
      const int k = B_KFAST ? e % kGemmBK : e / T::BN;
      const bool ok = ((okb >> p) & 1u) && (k0 + k < kend);
      const double v = fb(rb[p], k0 + k, j);
      sb[k * T::PB + j] = ok ? v : 0.0;
    }
  };

  fetch(kbeg);
  stash(kbeg, smem);
  if (kbeg + kGemmBK < kend) fetch(kbeg + kGemmBK);
  __syncthreads();
  int cur = 0;
  for (int k0 = kbeg; k0 < kend; k0 += kGemmBK) {
    const double* sa = smem + cur * T::kStageDoubles;
    const double* sb = sa + kGemmBK * T::PA;
    // next tile: registers -> the other LDS stage; tile after next: issue loads
    if (k0 + kGemmBK < kend) stash(k0 + kGemmBK, smem + (cur ^ 1) * T::kStageDoubles);
    if (k0 + 2 * kGemmBK < kend) fetch(k0 + 2 * kGemmBK);
    // fragments of k-step kk+1 are read while the MFMAs of k-step kk run (two register sets):
    // with few waves per SIMD nothing else would cover the LDS latency
    double a[2][TM], b[2][TN];
    auto frags = [&](int kk, int slot) {
      const int kr = kk + (lane >> 4);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) a[slot][tm] = sa[kr * T::PA + wm * 16 * TM + tm * 16 + (lane & 15)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) b[slot][tn] = sb[kr * T::PB + wn * 16 * TN + tn * 16 + (lane & 15)];
    };
    frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < kGemmBK; kk += 4) {
      const int slot = (kk >> 2) & 1;
      if (kk + 4 < kGemmBK) frags(kk + 4, slot ^ 1);
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[slot][tm], b[slot][tn], acc[tm][tn], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);   // the reads of the next k-step first
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);   // then this k-step's MFMAs
    }
    __syncthreads();  // stage cur free for the tile after next, stage cur^1 complete
    cur ^= 1;
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
