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
// The block lives in LDS and is processed in 16 x 16 sub-blocks.  For each
// diagonal sub-block one wave factors it and inverts the factor in registers
// (lane = row, pivots and multipliers passed around with v_readlane, no
// barriers); the sub-blocks below and the trailing sub-blocks are then updated
// with 16x16x4 float64 MFMAs by all four waves.  The inverse is built the same
// way, one wave per block column.  X is parked in the upper sub-blocks.
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
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nb = (s + 15) >> 4, sp = nb << 4;
  const int l16 = lane & 15, lq = lane >> 4;

  // load the lower triangle, sixteen independent loads per thread in flight
  for (int base = 0; base < sp * sp; base += 256 * 16) {
    double v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = base + tid + 256 * u;
      const int i = e / sp, j = e - i * sp;
      const bool ld = (e < sp * sp) & (i < s) & (j <= i);
      v[u] = G[ld ? (int64_t)(o + i) * n + o + j : (int64_t)o * n + o];
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int e = base + tid + 256 * u;
      const int i = e / sp, j = e - i * sp;
      const bool ld = (i < s) & (j <= i);
      if (e < sp * sp) S[i * kLeafP + j] = ld ? v[u] : ((i >= s && i == j) ? 1.0 : 0.0);  // padding: identity
    }
  }
  __syncthreads();

  for (int d = 0; d < nb; ++d) {
    const int b0 = 16 * d;
    if (wave == 0) {
      // ---- factor the diagonal sub-block and invert its factor (lanes 0..15)
      double a[16], id[16];
#pragma unroll
      for (int c = 0; c < 16; ++c) a[c] = S[(b0 + l16) * kLeafP + b0 + c];
      int bad = -1;
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        double p = lane_bcast(a[j], j);
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
        id[j] = r;
        a[j] = (l16 == j) ? sq : a[j] * r;
#pragma unroll
        for (int k = j + 1; k < 16; ++k) a[k] = fma(-a[j], lane_bcast(a[j], k), a[k]);
      }
      if (bad >= 0 && b0 + bad < s && tid == 0 && info[0] == PTQ_OK) {
        info[0] = PTQ_ERR_NOT_SPD;
        info[1] = n - 1 - (o + b0 + bad);
      }
      // column l16 of the inverse: x[i] = -(sum_{k<i} L_ik x[k]) / L_ii, x[l16] = 1 / L_ii
      double x[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        double sum = 0.0;
#pragma unroll
        for (int k = 0; k < i; ++k) sum = fma(lane_bcast(a[k], i), x[k], sum);
        x[i] = (l16 == i) ? id[i] : (l16 < i ? -sum * id[i] : 0.0);
      }
      if (lane < 16) {
#pragma unroll
        for (int c = 0; c < 16; ++c) {
          if (c <= lane) S[(b0 + lane) * kLeafP + b0 + c] = a[c];
          XD[(d * 16 + c) * kXdP + lane] = x[c];
        }
      }
    }
    __syncthreads();
    // ---- sub-blocks below the diagonal one: L_id = G_id X_dd^T
    for (int ib = d + 1 + wave; ib < nb; ib += 4) {
      f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const double av = S[(16 * ib + l16) * kLeafP + b0 + 4 * kk + lq];
        const double bv = XD[(d * 16 + l16) * kXdP + 4 * kk + lq];
        acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) S[(16 * ib + 4 * r + lq) * kLeafP + b0 + l16] = acc[r];
    }
    __syncthreads();
    // ---- trailing sub-blocks (ib >= jb > d): G_ij -= L_id L_jd^T
    {
      const int T = nb - 1 - d;
      const int cnt = T * (T + 1) / 2;
      for (int q = wave; q < cnt; q += 4) {
        int ii = 0, rem = q;
        while (rem > ii) {
          rem -= ii + 1;
          ++ii;
        }
        const int ib = d + 1 + ii, jb = d + 1 + rem;
        f64x4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const double av = S[(16 * ib + l16) * kLeafP + b0 + 4 * kk + lq];
          const double bv = S[(16 * jb + l16) * kLeafP + b0 + 4 * kk + lq];
          acc = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) S[(16 * ib + 4 * r + lq) * kLeafP + 16 * jb + l16] -= acc[r];
      }
    }
    __syncthreads();
  }

  // ---- inverse, one wave per block column jb:
  //   X_ij = -X_ii * sum_{k=jb}^{ib-1} L_ik X_kj ;  X_kj (k > jb) is kept in sub-block (jb, k)
  // block column jb costs about (nb - jb)^2 / 2 sub-block products: deal the columns to
  // the waves longest first, each to the least loaded wave
  int mine = 0;
  {
    int load[4] = {0, 0, 0, 0};
    for (int jb = 0; jb < nb; ++jb) {
      int w = 0;
      for (int c = 1; c < 4; ++c)
        if (load[c] < load[w]) w = c;
      load[w] += (nb - jb) * (nb - jb + 1);
      if (w == wave) mine |= 1 << jb;
    }
  }
  for (int jb = 0; jb < nb; ++jb) {
    if (!((mine >> jb) & 1)) continue;
    for (int ib = jb + 1; ib < nb; ++ib) {
      f64x4 t = {0.0, 0.0, 0.0, 0.0};
      for (int k = jb; k < ib; ++k) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const double av = S[(16 * ib + l16) * kLeafP + 16 * k + 4 * kk + lq];
          const double bv = (k == jb) ? XD[(jb * 16 + 4 * kk + lq) * kXdP + l16]
                                      : S[(16 * jb + 4 * kk + lq) * kLeafP + 16 * k + l16];
          t = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, t, 0, 0, 0);
        }
      }
      // the accumulator layout (row 4r + lane/16) is the B-fragment layout of k-step r
      f64x4 xo = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const double av = -XD[(ib * 16 + l16) * kXdP + 4 * kk + lq];
        xo = __builtin_amdgcn_mfma_f64_16x16x4f64(av, t[kk], xo, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) S[(16 * jb + 4 * r + lq) * kLeafP + 16 * ib + l16] = xo[r];
    }
  }
  __syncthreads();

  // X(i, j), i >= j, goes to U[n-1-(o+i)][n-1-(o+j)]
  for (int e = tid; e < sp * sp; e += 256) {
    const int i = e / sp, j = e - i * sp;
    if (i >= s || j > i) continue;
    const int ib = i >> 4, jb = j >> 4;
    const double x = (ib == jb) ? XD[(ib * 16 + (i & 15)) * kXdP + (j & 15)]
                                : S[(16 * jb + (i & 15)) * kLeafP + 16 * ib + (j & 15)];
    U[(int64_t)(n - 1 - (o + i)) * ldu + (n - 1 - (o + j))] = x;
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
  static constexpr bool A_KFAST = true, B_KFAST = true, REV_I = false, REV_J = true;
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
  static constexpr bool A_KFAST = false, B_KFAST = false, REV_I = false, REV_J = false;
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
  static constexpr bool A_KFAST = false, B_KFAST = false, REV_I = false, REV_J = false;
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
  static constexpr bool A_KFAST = true, B_KFAST = false, REV_I = true, REV_J = false;
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

template <int TM, int TN, class Op>
__device__ __forceinline__ void node_gemm_tile(const Op& op, int bx, int by, int gx, int gy, double* smem) {
  using T = DgemmTile<TM, TN>;
  // tiles with the longest k range first (triangular operands make them uneven)
  const int bi = Op::REV_I ? gy - 1 - by : by;
  const int bj = Op::REV_J ? gx - 1 - bx : bx;
  const int i0 = bi * T::BM, j0 = bj * T::BN;
  const int i1 = min(i0 + T::BM, op.M()), j1 = min(j0 + T::BN, op.N());
  if (!op.active(i0, i1, j0, j1)) return;
  int kb, ke;
  op.krange(i0, i1, j0, j1, kb, ke);
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  dgemm_mainloop<TM, TN, Op::A_KFAST, Op::B_KFAST>(acc, op.a(i0), DgemmIdentity{}, op.b(j0), DgemmIdentity{},
                                                   i1 - i0, j1 - j0, kb, ke, smem);
  dgemm_foreach(acc, [&](int i, int j, double v) { op.store(i0 + i, j0 + j, v); });
}

template <int TM, int TN, class Op>
__global__ __launch_bounds__(256) void node_gemm_kernel(Op op) {
  extern __shared__ double smem[];
  node_gemm_tile<TM, TN>(op, blockIdx.x, blockIdx.y, gridDim.x, gridDim.y, smem);
}

// Two independent steps in one launch: workgroups [0, gx1*gy1) take the tiles of the first.
template <int TM, int TN, class Op1, class Op2>
__global__ __launch_bounds__(256) void node_gemm2_kernel(Op1 op1, Op2 op2, int gx1, int gy1, int gx2, int gy2) {
  extern __shared__ double smem[];
  const int b = blockIdx.x, n1 = gx1 * gy1;
  if (b < n1)
    node_gemm_tile<TM, TN>(op1, b % gx1, b / gx1, gx1, gy1, smem);
  else
    node_gemm_tile<TM, TN>(op2, (b - n1) % gx2, (b - n1) / gx2, gx2, gy2, smem);
}

template <int TM, int TN, class Op>
void launch_tiles(const Op& op, int M, int N, hipStream_t st) {
  using T = DgemmTile<TM, TN>;
  static bool opted_in = false;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  if (!opted_in) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(node_gemm_kernel<TM, TN, Op>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    opted_in = true;
  }
  dim3 g((unsigned)ceil_div(N, T::BN), (unsigned)ceil_div(M, T::BM));
  node_gemm_kernel<TM, TN, Op><<<g, 256, lds, st>>>(op);
}

template <int TM, int TN, class Op1, class Op2>
void launch_tiles2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  using T = DgemmTile<TM, TN>;
  static bool opted_in = false;
  constexpr int lds = T::kSmemDoubles * (int)sizeof(double);
  if (!opted_in) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(node_gemm2_kernel<TM, TN, Op1, Op2>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    opted_in = true;
  }
  const int gx1 = (int)ceil_div(N1, T::BN), gy1 = (int)ceil_div(M1, T::BM);
  const int gx2 = (int)ceil_div(N2, T::BN), gy2 = (int)ceil_div(M2, T::BM);
  node_gemm2_kernel<TM, TN, Op1, Op2><<<(unsigned)(gx1 * gy1 + gx2 * gy2), 256, lds, st>>>(op1, op2, gx1, gy1, gx2, gy2);
}

// Tile shape by problem size: 64 x 128 once there are enough tiles to fill the chip several
// times over, 32 x 32 for the small nodes deep in the recursion (more workgroups, each with a
// short k loop: those launches are bound by latency, not by the matrix pipe), else 64 x 64.
inline int tile_class(int M, int N) {
  if (ceil_div(M, 64) * ceil_div(N, 128) >= 1024) return 2;
  if (ceil_div(M, 64) * ceil_div(N, 64) <= 64) return 0;
  return 1;
}

template <class Op>
void launch_node(const Op& op, int M, int N, hipStream_t st) {
  switch (tile_class(M, N)) {
    case 2: launch_tiles<2, 4, Op>(op, M, N, st); break;
    case 1: launch_tiles<2, 2, Op>(op, M, N, st); break;
    default: launch_tiles<1, 1, Op>(op, M, N, st); break;
  }
}

template <class Op1, class Op2>
void launch_node2(const Op1& op1, int M1, int N1, const Op2& op2, int M2, int N2, hipStream_t st) {
  const int c1 = tile_class(M1, N1), c2 = tile_class(M2, N2);
  switch (c1 < c2 ? c1 : c2) {
    case 2: launch_tiles2<2, 4, Op1, Op2>(op1, M1, N1, op2, M2, N2, st); break;
    case 1: launch_tiles2<2, 2, Op1, Op2>(op1, M1, N1, op2, M2, N2, st); break;
    default: launch_tiles2<1, 1, Op1, Op2>(op1, M1, N1, op2, M2, N2, st); break;
  }
}

void recurse(double* G, double* U, int ldu, int n, int o, int s, int32_t* info, hipStream_t st) {
  if (s <= kLeaf) {
    leaf_kernel<<<1, 256, kLeafLdsBytes, st>>>(G, n, o, s, U, ldu, info);
    return;
  }
  const int nb = (int)ceil_div(s, kLeaf);
  const int s1 = (nb / 2) * kLeaf;
  const int s2 = s - s1;
  Node nd{G, U, ldu, n, o, s1, s2};
  recurse(G, U, ldu, n, o, s1, info, st);
  launch_node(OpPanel{nd}, s2, s1, st);
  // the trailing update and T = L21 X11 both need only L21 and touch different blocks
  launch_node2(OpSyrk{nd}, s2, s2, OpT{nd}, s2, s1, st);
  recurse(G, U, ldu, n, o + s1, s2, info, st);
  launch_node(OpX21{nd}, s2, s1, st);
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
  static bool lds_opt_in = false;
  if (!lds_opt_in) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(leaf_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLeafLdsBytes) != hipSuccess)
      return PTQ_ERR_HIP;
    lds_opt_in = true;
  }
  diag_stats_kernel<<<1, 1024, 0, st>>>(H, ldh, (int)n, damp, dead_mask, scal, info);
  PTQ_HIP_CHECK_LAUNCH();
  dim3 g((unsigned)ceil_div(n, 256), (unsigned)n);
  build_work_kernel<<<g, 256, 0, st>>>(H, ldh, (int)n, scal, G, U, ldu);
  PTQ_HIP_CHECK_LAUNCH();
  recurse(G, U, (int)ldu, (int)n, 0, (int)n, info, st);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
