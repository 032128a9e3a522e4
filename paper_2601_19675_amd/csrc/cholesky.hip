// Damped Cholesky factor of the inverse Hessian:  U upper, U^T U = H_d^{-1}.
//
// Route.  With J the index reversal, G = J H_d J = L L^T (ordinary lower
// Cholesky) gives H_d = R R^T with R = J L J upper, hence H_d^{-1} = R^{-T} R^{-1}
// and U = R^{-1} = J L^{-1} J.  So one Cholesky factorization and one
// triangular inverse, both on the reversed matrix, and the result written back
// through the reversal.  Both are done by one recursion on the diagonal block
// [o, o+s) of G, which returns X = L^{-1} of that block:
//
//     split s = s1 + s2
//     X11           = rec(G11)
//     L21           = G21 X11^T                       (GEMM, X11 triangular)
//     G22          -= L21 L21^T                       (SYRK, lower tiles)  } one launch
//     T             = L21 X11                                              }
//     X22           = rec(G22)
//     X21           = -X22 T
//
// Every off-diagonal step is a float64 MFMA GEMM; only blocks of at most 128
// columns are factored and inverted inside one workgroup (in LDS).  L itself
// is never needed again, so only X is kept: it is stored directly in U through
// the reversal, X(i,j) = U[n-1-i][n-1-j].  L21^T is parked in the (otherwise
// unused) upper triangle of the work matrix, L21 X11 in the dead G21 block.
#include "dgemm.h"

#include <atomic>
#include <mutex>

namespace ptq {
namespace {

constexpr int kLeaf = 128;          // largest block factored inside one workgroup

// ---- diagonal statistics: dead channels, mean of the fixed diagonal ---------
__global__ __launch_bounds__(1024) void diag_stats_kernel(const double* __restrict__ H, int64_t ldh,
                                                          int n, double damp, uint8_t* dead_mask,
                                                          double* scal, int32_t* info) {
  __shared__ double part[1024];
  double s = 0.0;
  for (int j = threadIdx.x; j < n; j += 1024) {
    double d = H[(int64_t)j * ldh + j];
    const bool dead = (d == 0.0);
    if (dead) d = 1.0;
    if (dead_mask) dead_mask[j] = dead ? 1 : 0;
    s += d;
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    scal[0] = damp * (part[0] / (double)n);
    info[0] = PTQ_OK;
    info[1] = 0;
  }
}

// G = J H_d J (lower triangle, zeros above), and U cleared.
__global__ __launch_bounds__(256) void build_work_kernel(const double* __restrict__ H, int64_t ldh,
                                                         int n, const double* __restrict__ scal,
                                                         double* __restrict__ G, double* __restrict__ U,
                                                         int64_t ldu) {
  const int i = blockIdx.y;
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  double g = 0.0;
  if (j <= i) {
    const int hi = n - 1 - i, hj = n - 1 - j;  // hi <= hj: upper triangle of H
    g = H[(int64_t)hi * ldh + hj];
    if (i == j) {
      if (g == 0.0) g = 1.0;
      g += scal[0];
    }
  }
  G[(int64_t)i * n + j] = g;
  U[(int64_t)i * ldu + j] = 0.0;
}

// ---- leaf: X = inverse of the Cholesky factor of G[o:o+s, o:o+s], s <= 128 ---
// The block lives in LDS and is processed in 16 x 16 sub-blocks, right-looking.  Factoring a
// diagonal sub-block and inverting its factor is a chain of dependent operations that one
// wave does in registers (lane = row, pivots and multipliers passed around with v_readlane,
// no barriers); everything else is 16x16x4 float64 MFMA work on sub-blocks.  The chain is the
// critical path, so the steps are skewed: while wave 0 factors diagonal block d+1 (after
// applying step d's update to it itself), the other waves apply the rest of step d's trailing
// update and pre-compute row d+1 of the inverse.
//
//   P1(d)  all waves   L_id = G_id X_dd^T  (i > d);   X_dj = -X_dd T_dj  (j < d)
//   P2(d)  wave 0      G_{d+1,d+1} -= L_{d+1,d} L_{d+1,d}^T ;  factor + invert it -> X_{d+1,d+1}
//          waves 1-3   G_ij -= L_id L_jd^T  (i >= j > d, all but (d+1,d+1));
//                      T_{d+1,j} = sum_{k=j..d} L_{d+1,k} X_kj  (j <= d)
//
// X_ij (i > j) and before it T_ij are parked in the unused upper sub-block (j, i); the
// inverses of the diagonal sub-blocks have their own array.
__device__ __forceinline__ double lane_bcast(double v, int src) {
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), src);
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), src);
  return __hiloint2double(hi, lo);
}

constexpr int kLeafP = kLeaf + 1;   // pitch of the LDS block
constexpr int kXdP = 17;            // pitch of a stored 16 x 16 diagonal inverse
constexpr size_t kLeafLdsBytes = (size_t)(kLeaf * kLeafP + (kLeaf / 16) * 16 * kXdP) * sizeof(double);

__global__ __launch_bounds__(256) void leaf_kernel(const double* __restrict__ G, int n, int o, int s,
                                                   double* __restrict__ U, int64_t ldu, int32_t* info) {
  extern __shared__ double lds[];
  double* S = lds;                      // [128][129]
  double* XD = lds + kLeaf * kLeafP;    // [8][16][17] inverses of the diagonal sub-blocks
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: keeps the work-list arithmetic scalar
  const int nb = (s + 15) >> 4, sp = nb << 4;
  const int l16 = lane & 15, lq = lane >> 4;

  // load the lower triangle: thread = (column j, row parity), all its loads in flight at once
  // (padding rows / columns beyond s: identity)
  {
    const int j = tid & 127, i0 = tid >> 7;
    double v[kLeaf / 2];
#pragma unroll
    for (int u = 0; u < kLeaf / 2; ++u) {
      const int i = i0 + 2 * u;
      const bool ld = (i < s) & (j <= i);
      v[u] = ld ? G[(int64_t)(o + i) * n + o + j] : ((i == j) ? 1.0 : 0.0);
    }
#pragma unroll
    for (int u = 0; u < kLeaf / 2; ++u) {
      const int i = i0 + 2 * u;
      if (i < sp && j < sp) S[i * kLeafP + j] = v[u];
    }
  }
  __syncthreads();

  // Factor diagonal sub-block d and invert its factor, one wave, all 64 lanes.  The symmetric
  // 16 x 16 block M sits in four registers per lane in the accumulator layout of the MFMA read
  // through the symmetry: lane (lq, l16), register r holds M(l16, 4 r + lq).  Column group g
  // (columns 4g .. 4g+3) is then register g, and that register is at once the A and the B
  // fragment of the 16 x 4 panel, so the rank-4 update of the later column groups is one MFMA
  // with no data movement.  Inside a group the pivots go one by one: the pivot column is
  // handed to the other lane groups with two lane permutes.  With `update`, step d-1's
  // contribution L_{d,d-1} L_{d,d-1}^T is taken off the block first.
  // The inverse follows by block forward substitution with 4 x 4 blocks: the four diagonal
  // 4 x 4 inverses are computed from broadcast entries, then per block row two MFMAs:
  // X_h = D_h - Dinv_h (T_h),  T += L(:, h) X_h.
  auto factor_diag = [&](int d, bool update) {
    const int b0 = 16 * d;
    double m[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int c = 4 * r + lq;
      const int hi = l16 > c ? l16 : c, lo = l16 > c ? c : l16;
      m[r] = S[(b0 + hi) * kLeafP + b0 + lo];
    }
    if (update) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const double lv = S[(b0 + l16) * kLeafP + b0 - 16 + 4 * kk + lq];
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(lv, lv, acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) m[r] -= acc[r];
    }
    auto lane_fetch = [&](double v, int src_lane) -> double {  // per-lane source (ds_bpermute)
      const int lo = __builtin_amdgcn_ds_bpermute(src_lane << 2, __double2loint(v));
      const int hi = __builtin_amdgcn_ds_bpermute(src_lane << 2, __double2hiint(v));
      return __hiloint2double(hi, lo);
    };
    int bad = -1;
    double rinv[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int j = 4 * g + k;
        double p = lane_bcast(m[g], 16 * k + j);
        if (!(p > 0.0)) {
          if (bad < 0) bad = j;
          p = 1.0;
        }
        // 1/sqrt(p) by two Newton steps on the hardware estimate, then one
        // correction each for sqrt(p) and its reciprocal (no division, no sqrt call)
        const double h = 0.5 * p;
        double r = __builtin_amdgcn_rsq(p);
        r = r * fma(-h * r, r, 1.5);
        r = r * fma(-h * r, r, 1.5);
        double sq = p * r;
        sq = fma(fma(-sq, sq, p), 0.5 * r, sq);
        r = fma(fma(-sq, r, 1.0), r, r);
        rinv[j] = r;
        const double colv = (l16 == j) ? sq : (l16 > j ? m[g] * r : 0.0);
        m[g] = (lq == k) ? colv : m[g];
        if (k < 3) {
          const double cj = lane_fetch(m[g], 16 * k + l16);          // L(own row, j)
          const double mu = lane_fetch(m[g], 16 * k + 4 * g + lq);   // L(own column, j)
          m[g] = (lq > k) ? fma(-cj, mu, m[g]) : m[g];
        }
      }
      if (g < 3) {
        const f64x4 acc = __builtin_amdgcn_mfma_f64_16x16x4f64(m[g], m[g], f64x4{0.0, 0.0, 0.0, 0.0}, 0, 0, 0);
#pragma unroll
        for (int r = g + 1; r < 4; ++r) m[r] -= acc[r];
      }
    }
    if (bad >= 0 && b0 + bad < s && lane == 0 && info[0] == PTQ_OK) {
      info[0] = PTQ_ERR_NOT_SPD;
      info[1] = n - 1 - (o + b0 + bad);
    }
    // diagonal 4 x 4 inverses: dA[h] = Dinv(:, 4h..4h+3) as an A fragment (lane (lq, l16) holds
    // x_ab with a = l16 - 4h, b = lq), dD[h] the same block in the accumulator layout
    double dA[4], dD[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const double l10 = lane_bcast(m[h], 4 * h + 1), l20 = lane_bcast(m[h], 4 * h + 2);
      const double l30 = lane_bcast(m[h], 4 * h + 3), l21 = lane_bcast(m[h], 16 + 4 * h + 2);
      const double l31 = lane_bcast(m[h], 16 + 4 * h + 3), l32 = lane_bcast(m[h], 32 + 4 * h + 3);
      const double r0 = rinv[4 * h], r1 = rinv[4 * h + 1], r2 = rinv[4 * h + 2], r3 = rinv[4 * h + 3];
      const double x10 = -r1 * (l10 * r0);
      const double x21 = -r2 * (l21 * r1);
      const double x32 = -r3 * (l32 * r2);
      const double x20 = -r2 * fma(l21, x10, l20 * r0);
      const double x31 = -r3 * fma(l32, x21, l31 * r1);
      const double x30 = -r3 * fma(l32, x20, fma(l31, x10, l30 * r0));
      const int a = l16 - 4 * h, bq = lq;
      double v = 0.0;
      v = (a == 0 && bq == 0) ? r0 : v;
      v = (a == 1 && bq == 1) ? r1 : v;
      v = (a == 2 && bq == 2) ? r2 : v;
      v = (a == 3 && bq == 3) ? r3 : v;
      v = (a == 1 && bq == 0) ? x10 : v;
      v = (a == 2 && bq == 1) ? x21 : v;
      v = (a == 3 && bq == 2) ? x32 : v;
      v = (a == 2 && bq == 0) ? x20 : v;
      v = (a == 3 && bq == 1) ? x31 : v;
      v = (a == 3 && bq == 0) ? x30 : v;
      dA[h] = v;
      // accumulator layout: lane (lq = a', l16 = 4h + b') wants x_{a'b'}, held by lane (b', 4h + a')
      const int bp = l16 - 4 * h;
      const bool in = (bp >= 0) & (bp < 4);
      const double t = lane_fetch(v, in ? 16 * bp + 4 * h + lq : lane);
      dD[h] = in ? t : 0.0;
    }
    f64x4 T = {0.0, 0.0, 0.0, 0.0};
    double X[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      if (h > 0) {
        const f64x4 o = __builtin_amdgcn_mfma_f64_16x16x4f64(dA[h], T[h], f64x4{0.0, 0.0, 0.0, 0.0}, 0, 0, 0);
        X[h] = dD[h] - o[h];
      } else {
        X[h] = dD[h];
      }
      if (h < 3) T = __builtin_amdgcn_mfma_f64_16x16x4f64(m[h], X[h], T, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) XD[(d * 16 + 4 * r + lq) * kXdP + l16] = X[r];
  };
  auto fragA = [&](const double* blk, int kk) { return blk[l16 * kLeafP + 4 * kk + lq]; };

  if (wave == 0) factor_diag(0, false);
  __syncthreads();

  for (int d = 0; d < nb; ++d) {
    const int b0 = 16 * d;
    // ---- P1: column d of L below the diagonal, row d of the inverse left of it
    {
      const int nB = nb - 1 - d, nItems = nB + d;
      for (int q = wave; q < nItems; q += 4) {
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
        if (q < nB) {
          const int ib = d + 1 + q;  // wave 0 gets ib = d + 1, which it needs first in P2
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            const double av = fragA(S + (16 * ib) * kLeafP + b0, kk);
            const double bv = XD[(d * 16 + l16) * kXdP + 4 * kk + lq];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) S[(16 * ib + 4 * r + lq) * kLeafP + b0 + l16] = acc[r];
        } else {
          const int jb = q - nB;  // X_dj = -X_dd T_dj, in place in the parked block (jb, d)
          double* blk = S + (16 * jb) * kLeafP + b0;
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            const double av = -XD[(d * 16 + l16) * kXdP + 4 * kk + lq];
            const double bv = blk[(4 * kk + lq) * kLeafP + l16];
            acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) blk[(4 * r + lq) * kLeafP + l16] = acc[r];
        }
      }
    }
    __syncthreads();
    if (d + 1 >= nb) break;
    // ---- P2
    if (wave == 0) {
      factor_diag(d + 1, true);
    } else {
      // row d+1 of the inverse, longest sums first: T_{d+1,j} = sum_{k=j..d} L_{d+1,k} X_kj
      // (two accumulators, so that consecutive k blocks do not wait for each other)
      const int ib = d + 1;
      for (int jb = wave - 1; jb <= d; jb += 3) {
        f64x4 t0 = {0.0, 0.0, 0.0, 0.0}, t1 = {0.0, 0.0, 0.0, 0.0};
        for (int k = jb; k <= d; k += 2) {
          const bool two = k + 1 <= d;
          const int k1 = two ? k + 1 : k;
          double av0[4], bv0[4], av1[4], bv1[4];
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            av0[kk] = fragA(S + (16 * ib) * kLeafP + 16 * k, kk);
            bv0[kk] = (k == jb) ? XD[(jb * 16 + 4 * kk + lq) * kXdP + l16]
                                : S[(16 * jb + 4 * kk + lq) * kLeafP + 16 * k + l16];
            av1[kk] = fragA(S + (16 * ib) * kLeafP + 16 * k1, kk);
            bv1[kk] = S[(16 * jb + 4 * kk + lq) * kLeafP + 16 * k1 + l16];
          }
#pragma unroll
          for (int kk = 0; kk < 4; ++kk) {
            t0 = __builtin_amdgcn_mfma_f64_16x16x4f64(av0[kk], bv0[kk], t0, 0, 0, 0);
            t1 = __builtin_amdgcn_mfma_f64_16x16x4f64(av1[kk], two ? bv1[kk] : 0.0, t1, 0, 0, 0);
          }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) S[(16 * jb + 4 * r + lq) * kLeafP + 16 * ib + l16] = t0[r] + t1[r];
      }
      // trailing sub-blocks (i2 >= j2 > d), triangular index 1 .. cnt-1 (index 0 = (d+1, d+1) is
      // wave 0's), dealt round-robin after the d+1 sums above and processed two at a time
      const int T = nb - 1 - d;
      const int cnt = T * (T + 1) / 2;
      int c0 = (wave - 1 - d) % 3;
      if (c0 < 0) c0 += 3;
      if (c0 == 0) c0 = 3;
      // (ii, rem) = row / column of triangular index c, advanced incrementally (index += 3)
      int ii = 0, rem = c0;
      auto settle = [&]() {
        while (rem > ii) {
          rem -= ii + 1;
          ++ii;
        }
      };
      for (int c = c0; c < cnt; c += 6) {
        const bool two = c + 3 < cnt;
        settle();
        const int ia = d + 1 + ii, ja = d + 1 + rem;
        int ib2 = ia, jb2 = ja;
        rem += 3;
        if (two) {
          settle();
          ib2 = d + 1 + ii;
          jb2 = d + 1 + rem;
        }
        rem += 3;
        double a0[4], b0v[4], a1[4], b1[4], cur0[4], cur1[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          a0[kk] = fragA(S + (16 * ia) * kLeafP + b0, kk);
          b0v[kk] = fragA(S + (16 * ja) * kLeafP + b0, kk);
          a1[kk] = fragA(S + (16 * ib2) * kLeafP + b0, kk);
          b1[kk] = fragA(S + (16 * jb2) * kLeafP + b0, kk);
          cur0[kk] = S[(16 * ia + 4 * kk + lq) * kLeafP + 16 * ja + l16];
          cur1[kk] = S[(16 * ib2 + 4 * kk + lq) * kLeafP + 16 * jb2 + l16];
        }
        f64x4 acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a0[kk], b0v[kk], acc0, 0, 0, 0);
          acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a1[kk], b1[kk], acc1, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) S[(16 * ia + 4 * r + lq) * kLeafP + 16 * ja + l16] = cur0[r] - acc0[r];
        if (two) {
#pragma unroll
          for (int r = 0; r < 4; ++r) S[(16 * ib2 + 4 * r + lq) * kLeafP + 16 * jb2 + l16] = cur1[r] - acc1[r];
        }
      }
    }
    __syncthreads();
  }

  // X(i, j), i >= j, goes to U[n-1-(o+i)][n-1-(o+j)]: thread = (column j, row parity)
  {
    const int j = tid & 127, i0 = tid >> 7, jb = j >> 4;
    double* urow = U + (int64_t)(n - 1 - o) * ldu + (n - 1 - (o + j));
#pragma unroll 8
    for (int u = 0; u < kLeaf / 2; ++u) {
      const int i = i0 + 2 * u;
      if (i < s && j <= i) {
        const int ib = i >> 4;
        const double x = (ib == jb) ? XD[(ib * 16 + (i & 15)) * kXdP + (j & 15)]
                                    : S[(16 * jb + (i & 15)) * kLeafP + 16 * ib + (j & 15)];
        urow[-(int64_t)i * ldu] = x;
      }
    }
  }
}

// ---- the four GEMM steps of one recursion node -------------------------------
// Each step describes its operands as strided views for the tile at (i0, j0):
// A(i, k) and B(k, j) with i, j tile-local and k counted from the block start.
struct Node {
  double* G;      // work matrix, n x n, ld = n
  double* U;      // output, X reversed: X(i, j) = U[n-1-i][n-1-j]
  int ldu;
  int n, o, s1, s2;
  __device__ __forceinline__ const double* g(int i, int j) const { return G + (int64_t)i * n + j; }
  __device__ __forceinline__ const double* x(int i, int j) const {
    return U + (int64_t)(n - 1 - i) * ldu + (n - 1 - j);
  }
};

// L21 = G21 X11^T, stored transposed in the mirror block of G.
struct OpPanel {
  static constexpr bool A_KFAST = true, B_KFAST = true;
  static constexpr int K_ORDER = +2;  // k range grows with the column tile: last column tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int, int, int j1, int& kb, int& ke) const { kb = 0; ke = min(nd.s1, j1); }
  __device__ DView a(int i0) const { return DView{nd.g(nd.o + nd.s1 + i0, nd.o), nd.n, 1}; }
  __device__ DView b(int j0) const { return DView{nd.x(nd.o + j0, nd.o), -nd.ldu, -1}; }  // X11(j, k)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1) nd.G[(int64_t)(nd.o + j) * nd.n + nd.o + nd.s1 + i] = v;
  }
};

// G22 -= L21 L21^T on the lower triangle.
struct OpSyrk {
  static constexpr bool A_KFAST = false, B_KFAST = false;
  static constexpr int K_ORDER = 0;   // every active tile has the full k range
  static constexpr bool LOWER_ONLY = true;  // only tiles that touch the lower triangle are launched
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s2; }
  __device__ bool active(int, int i1, int j0, int) const { return i1 > j0; }
  __device__ void krange(int, int, int, int, int& kb, int& ke) const { kb = 0; ke = nd.s1; }
  __device__ DView a(int i0) const { return DView{nd.g(nd.o, nd.o + nd.s1 + i0), 1, nd.n}; }  // L21(i, k)
  __device__ DView b(int j0) const { return DView{nd.g(nd.o, nd.o + nd.s1 + j0), 1, nd.n}; }  // L21(j, k)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j <= i) nd.G[(int64_t)(nd.o + nd.s1 + i) * nd.n + nd.o + nd.s1 + j] -= v;
  }
};

// T = L21 X11, stored in the dead G21 block.
struct OpT {
  static constexpr bool A_KFAST = false, B_KFAST = false;
  static constexpr int K_ORDER = -2;  // k range shrinks with the column tile: first column tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int, int j0, int, int& kb, int& ke) const { kb = j0; ke = nd.s1; }
  __device__ DView a(int i0) const { return DView{nd.g(nd.o, nd.o + nd.s1 + i0), 1, nd.n}; }
  __device__ DView b(int j0) const { return DView{nd.x(nd.o, nd.o + j0), -1, -nd.ldu}; }  // X11(k, j)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1) nd.G[(int64_t)(nd.o + nd.s1 + i) * nd.n + nd.o + j] = v;
  }
};

// X21 = -X22 T.
struct OpX21 {
  static constexpr bool A_KFAST = true, B_KFAST = false;
  static constexpr int K_ORDER = +1;  // k range grows with the row tile: last row tile first
  static constexpr bool LOWER_ONLY = false;
  Node nd;
  __device__ int M() const { return nd.s2; }
  __device__ int N() const { return nd.s1; }
  __device__ bool active(int, int, int, int) const { return true; }
  __device__ void krange(int, int i1, int, int, int& kb, int& ke) const { kb = 0; ke = min(nd.s2, i1); }
  __device__ DView a(int i0) const {  // X22(i, k)
    return DView{nd.x(nd.o + nd.s1 + i0, nd.o + nd.s1), -nd.ldu, -1};
  }
  __device__ DView b(int j0) const { return DView{nd.g(nd.o + nd.s1, nd.o + j0), 1, nd.n}; }  // T(k, j)
  __device__ void store(int i, int j, double v) const {
    if (i < nd.s2 && j < nd.s1)
      nd.U[(int64_t)(nd.n - 1 - (nd.o + nd.s1 + i)) * nd.ldu + (nd.n - 1 - (nd.o + j))] = -v;
  }
};

// Column tiles of row tile bi that reach the lower triangle (square matrix, tile BM x BN).
template <int TM, int TN>
__host__ __device__ inline int lower_tiles_in_row(int bi, int gx) {
  const int c = ((bi + 1) * 32 * TM - 1) / (32 * TN) + 1;
  return c < gx ? c : gx;
}
template <int TM, int TN>
inline int lower_tiles(int gx, int gy) {
  int s = 0;
  for (int bi = 0; bi < gy; ++bi) s += lower_tiles_in_row<TM, TN>(bi, gx);
  return s;
}

// Tile `lin` of the gx x gy tile grid of a step.  Triangular operands make the k ranges uneven, so
// the tiles are handed out longest first, over the whole grid: the index the k range depends on
// (K_ORDER: +-1 row tile, +-2 column tile; sign = which end is longest) is the slow one.
template <int TM, int TN, class Op>
__device__ __forceinline__ void node_gemm_tile(const Op& op, int lin, int gx, int gy, double* smem) {
  using T = DgemmTile<TM, TN>;
  int bi, bj;
  if (Op::LOWER_ONLY) {
    // row tile bi has lower_tiles_in_row(bi) tiles (bj = 0 ..); rows from the last one up
    bi = gy - 1;
    int c = lower_tiles_in_row<TM, TN>(bi, gx);
    while (lin >= c) {
      lin -= c;
      --bi;
      c = lower_tiles_in_row<TM, TN>(bi, gx);
    }
    bj = lin;
  } else if (Op::K_ORDER == 2 || Op::K_ORDER == -2) {
    const int q = lin / gy;
    bi = lin - q * gy;
    bj = Op::K_ORDER > 0 ? gx - 1 - q : q;
  } else {
    const int q = lin / gx;
    bj = lin - q * gx;
    bi = Op::K_ORDER > 0 ? gy - 1 - q : q;
  }
  const int i0 = bi * T::BM, j0 = bj * T::BN;
  const int i1 = min(i0 + T::BM, op.M()), j1 = min(j0 + T::BN, op.N());
  if (!op.active(i0, i1, j0, j1)) return;
  int kb, ke;
  op.krange(i0, i1, j0, j1, kb, ke);
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  // a tile with no ragged edge takes the software-pipelined loop (same sums in the same order)
  // (its buffer loads address a tile's footprint with 32-bit byte offsets)
  const DView va = op.a(i0), vb = op.b(j0);
  const int64_t spana = ((int64_t)T::BM * abs(va.so) + (int64_t)(ke - kb) * abs(va.sk)) * 8;
  const int64_t spanb = ((int64_t)T::BN * abs(vb.so) + (int64_t)(ke - kb) * abs(vb.sk)) * 8;
  const bool full = (i1 - i0 == T::BM) && (j1 - j0 == T::BN) && ke > kb && ((ke - kb) % kGemmBK == 0) &&
                    spana < ((int64_t)1 << 31) && spanb < ((int64_t)1 << 31);
  bool done = false;
  if constexpr (TM * TN >= 4) {
    if (full) {
      dgemm_mainloop_pipelined<TM, TN, Op::A_KFAST, Op::B_KFAST>(acc, va, vb, kb, ke, smem);
      done = true;
    }
  }
  if (!done)
    dgemm_mainloop<TM, TN, Op::A_KFAST, Op::B_KFAST>(acc, va, DgemmIdentity{}, vb, DgemmIdentity{}, i1 - i0, j1 - j0,
                                                     kb, ke, smem);
  dgemm_foreach(acc, [&](int i, int j, double v) { op.store(i0 + i, j0 + j, v); });
}

// (64 x 64 tiles: three workgroups per CU, so the registers are capped for three; the 128 x 128 tile
// keeps 128 accumulator registers and two sets of staging registers and runs one or two per CU)
template <int TM, int TN, class Op>
__global__ __launch_bounds__(256, (TM * TN == 4) ? 3 : 1) void node_gemm_kernel(Op op, int gx, int gy, int total) {
  extern __shared__ double smem[];
  // one tile per workgroup, or, launched with fewer workgroups than tiles, a stride over the tile list
  // (both tile loops end with a barrier, so the LDS stages are free when the next tile starts)
  for (int lin = blockIdx.x; lin < total; lin += gridDim.x) node_gemm_tile<TM, TN>(op, lin, gx, gy, smem);
}

// Two independent steps in one launch: workgroups [0, n1) take the tiles of the first.
template <int TM, int TN, class Op1, class Op2>
__global__ __launch_bounds__(256, (TM * TN == 4) ? 3 : 1) void node_gemm2_kernel(Op1 op1, Op2 op2, int n1, int gx1, int gy1, int gx2, int gy2) {
  extern __shared__ double smem[];
  const int b = blockIdx.x;
  if (b < n1)
    node_gemm_tile<TM, TN>(op1, b, gx1, gy1, smem);
  else
    node_gemm_tile<TM, TN>(op2, b - n1, gx2, gy2, smem);
}

// max_wgs > 0 caps the number of workgroups (the tiles are then taken in a stride): used for work that
// runs beside the critical chain on a second stream and must leave compute units free for it
template <int TM, int TN, class Op>
bool launch_tiles(const Op& op, int M, int N, hipStream_t st, int max_wgs = 0) {
  using T = DgemmTile<TM, TN>;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  if (!lds_opt_in<node_gemm_kernel<TM, TN, Op>>(lds)) return false;
  const int gx = (int)ceil_div(N, T::BN), gy = (int)ceil_div(M, T::BM);
  const int total = Op::LOWER_ONLY ? lower_tiles<TM, TN>(gx, gy) : gx * gy;
  const int nwg = (max_wgs > 0 && max_wgs < total) ? max_wgs : total;
  node_gemm_kernel<TM, TN, Op><<<(unsigned)nwg, 256, lds, st>>>(op, gx, gy, total);
  return true;
}

template <int TM, int TN, class Op1, class Op2>
bool launch_tiles2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  using T = DgemmTile<TM, TN>;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  if (!lds_opt_in<node_gemm2_kernel<TM, TN, Op1, Op2>>(lds)) return false;
  const int gx1 = (int)ceil_div(N1, T::BN), gy1 = (int)ceil_div(M1, T::BM);
  const int gx2 = (int)ceil_div(N2, T::BN), gy2 = (int)ceil_div(M2, T::BM);
  const int n1 = Op1::LOWER_ONLY ? lower_tiles<TM, TN>(gx1, gy1) : gx1 * gy1;
  const int n2 = Op2::LOWER_ONLY ? lower_tiles<TM, TN>(gx2, gy2) : gx2 * gy2;
  node_gemm2_kernel<TM, TN, Op1, Op2><<<(unsigned)(n1 + n2), 256, lds, st>>>(op1, op2, n1, gx1, gy1, gx2, gy2);
  return true;
}

// Tile shape by problem size, as measured: 128 x 128 once there are enough tiles to fill the
// chip twice over; up to about a 1500-wide node 32 x 32 tiles (there the k loops are short and
// bound by the latency of their loads, whatever the tile: many small workgroups hide it best);
// 64 x 64 between.
inline int tile_class(int M, int N) {
  if (ceil_div(M, 128) * ceil_div(N, 128) >= 512) return 2;
  if (ceil_div(M, 64) * ceil_div(N, 64) <= 512) return 0;
  return 1;
}

template <class Op>
bool launch_node(const Op& op, int M, int N, hipStream_t st, int max_cus = 0) {
  switch (tile_class(M, N)) {
    case 2: return launch_tiles<4, 4, Op>(op, M, N, st, max_cus);          // one workgroup per compute unit
    case 1: return launch_tiles<2, 2, Op>(op, M, N, st, 3 * max_cus);      // three
    default: return launch_tiles<1, 1, Op>(op, M, N, st, 4 * max_cus);
  }
}

template <class Op1, class Op2>
bool launch_node2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  const int c1 = tile_class(M1, N1), c2 = tile_class(M2, N2);
  switch (c1 < c2 ? c1 : c2) {
    case 2: return launch_tiles2<4, 4, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
    case 1: return launch_tiles2<2, 2, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
    default: return launch_tiles2<1, 1, Op1, Op2>(op1, M1, N1, op2, M2, N2, st);
  }
}

// ---- a second stream for work that is off the critical chain ---------------------------------
// After the trailing update of a node the chain  leaf -> panel -> update -> leaf ...  of its second
// half is a sequence of small, latency-bound launches that leaves most of the chip idle, while
// T = L21 X11  of the node (a quarter of its flops) is needed only by the node's last step.  For the
// largest nodes (128 x 128 tiles) T therefore runs on a helper stream, forked after the update and
// joined before  X21 = -X22 T,  with at most kSideCus workgroups, so that the launches of the chain
// always find free compute units (measured at n = 11008: 128 gives the shortest total; 256 gains
// nothing, 64 makes T the longer path).  Smaller nodes gain nothing (measured) and keep T in the
// update's launch.  One helper stream and a few events per device, created on first use and kept
// for the life of the process (default priority).
constexpr int kSideCus = 128;
constexpr int kMaxDepth = 12;
struct Side {
  std::mutex lock;   // the events are reused call after call: one caller at a time enqueues a factor
  hipStream_t stream = nullptr;
  hipEvent_t fork[kMaxDepth], join[kMaxDepth];
  bool ok = false;
};

Side* side_for_device() {
  constexpr int kMaxDevices = 64;
  static Side sides[kMaxDevices];
  static std::atomic<int> state[kMaxDevices];   // 0 = untried, 1 = being set up, 2 = ready, 3 = unavailable
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  int expected = 0;
  if (state[dev].compare_exchange_strong(expected, 1)) {
    Side& sd = sides[dev];
    bool ok = hipStreamCreateWithFlags(&sd.stream, hipStreamNonBlocking) == hipSuccess;
    for (int d = 0; ok && d < kMaxDepth; ++d)
      ok = hipEventCreateWithFlags(&sd.fork[d], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&sd.join[d], hipEventDisableTiming) == hipSuccess;
    sd.ok = ok;
    state[dev].store(ok ? 2 : 3, std::memory_order_release);
  }
  while (state[dev].load(std::memory_order_acquire) == 1) {
  }
  return state[dev].load(std::memory_order_acquire) == 2 ? &sides[dev] : nullptr;
}

bool recurse(double* G, double* U, int ldu, int n, int o, int s, int32_t* info, hipStream_t st, Side* side, int depth) {
  if (s <= kLeaf) {
    leaf_kernel<<<1, 256, kLeafLdsBytes, st>>>(G, n, o, s, U, ldu, info);
    return true;
  }
  const int nb = (int)ceil_div(s, kLeaf);
  const int s1 = (nb / 2) * kLeaf;
  const int s2 = s - s1;
  Node nd{G, U, ldu, n, o, s1, s2};
  if (!recurse(G, U, ldu, n, o, s1, info, st, side, depth + 1) || !launch_node(OpPanel{nd}, s2, s1, st)) return false;
  // the trailing update and T = L21 X11 both need only L21 and touch different blocks
  if (side && depth < kMaxDepth && tile_class(s2, s1) == 2) {
    // a large node: the trailing update first, with the whole chip; then T beside the chain of the
    // second half (fork after the update, join before X21)
    if (!launch_node(OpSyrk{nd}, s2, s2, st)) return false;
    if (hipEventRecord(side->fork[depth], st) != hipSuccess ||
        hipStreamWaitEvent(side->stream, side->fork[depth], 0) != hipSuccess)
      return false;
    if (!launch_node(OpT{nd}, s2, s1, side->stream, kSideCus)) return false;
    if (hipEventRecord(side->join[depth], side->stream) != hipSuccess) return false;
    if (!recurse(G, U, ldu, n, o + s1, s2, info, st, side, depth + 1)) return false;
    if (hipStreamWaitEvent(st, side->join[depth], 0) != hipSuccess) return false;
    return launch_node(OpX21{nd}, s2, s1, st);
  }
  return launch_node2(OpSyrk{nd}, s2, s2, OpT{nd}, s2, s1, st) &&
         recurse(G, U, ldu, n, o + s1, s2, info, st, side, depth + 1) && launch_node(OpX21{nd}, s2, s1, st);
}

}  // namespace

size_t cholesky_workspace_bytes(int64_t n) {
  return align_up((size_t)n * (size_t)n * sizeof(double), 256) + 256;
}

ptq_status cholesky_launch(const double* H, int64_t ldh, int64_t n, double damp, double* U, int64_t ldu,
                           uint8_t* dead_mask, int32_t* info, void* ws, size_t ws_bytes,
                           hipStream_t st) {
  if (n == 0) return PTQ_OK;
  if (ws_bytes < cholesky_workspace_bytes(n)) return PTQ_ERR_WORKSPACE;
  double* G = static_cast<double*>(ws);
  double* scal = reinterpret_cast<double*>(static_cast<char*>(ws) +
                                           align_up((size_t)n * (size_t)n * sizeof(double), 256));
  if (!lds_opt_in<leaf_kernel>((int)kLeafLdsBytes)) return PTQ_ERR_HIP;
  diag_stats_kernel<<<1, 1024, 0, st>>>(H, ldh, (int)n, damp, dead_mask, scal, info);
  PTQ_HIP_CHECK_LAUNCH();
  dim3 g((unsigned)ceil_div(n, 256), (unsigned)n);
  build_work_kernel<<<g, 256, 0, st>>>(H, ldh, (int)n, scal, G, U, ldu);
  PTQ_HIP_CHECK_LAUNCH();
  // the helper stream only where a node is large enough to use it (the top node is the largest)
  const int top1 = (int)(ceil_div(n, kLeaf) / 2) * kLeaf;
  Side* side = (n > kLeaf && tile_class((int)n - top1, top1) == 2) ? side_for_device() : nullptr;
  bool ok;
  if (side) {
    std::lock_guard<std::mutex> hold(side->lock);
    ok = recurse(G, U, (int)ldu, (int)n, 0, (int)n, info, st, side, 0);
  } else {
    ok = recurse(G, U, (int)ldu, (int)n, 0, (int)n, info, st, nullptr, 0);
  }
  if (!ok) return PTQ_ERR_HIP;
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
