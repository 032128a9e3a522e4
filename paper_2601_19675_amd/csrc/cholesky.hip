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
//     G22          -= L21 L21^T                       (SYRK, lower tiles)
//     X22           = rec(G22)
//     X21           = -X22 (L21 X11)                  (two GEMMs)
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
constexpr int kLeafPitch = kLeaf + 1;
constexpr int kLeafThreads = 1024;

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
__global__ __launch_bounds__(kLeafThreads) void leaf_kernel(const double* __restrict__ G, int n, int o,
                                                            int s, double* __restrict__ U, int64_t ldu,
                                                            int32_t* info) {
  extern __shared__ double lds[];
  double* S = lds;                          // s x s, pitch 129: lower = L, strict upper = X^T
  double* invd = lds + kLeaf * kLeafPitch;  // 1 / L_jj
  const int tid = threadIdx.x;

  for (int e = tid; e < s * s; e += kLeafThreads) {
    const int i = e / s, j = e % s;
    S[i * kLeafPitch + j] = (j <= i) ? G[(int64_t)(o + i) * n + o + j] : 0.0;
  }
  __syncthreads();

  // right-looking factorization, one column at a time
  const int ti = tid >> 5, tk = tid & 31;
  for (int j = 0; j < s; ++j) {
    if (tid == 0) {
      double p = S[j * kLeafPitch + j];
      if (!(p > 0.0)) {
        if (info[0] == PTQ_OK) {
          info[0] = PTQ_ERR_NOT_SPD;
          info[1] = n - 1 - (o + j);
        }
        p = 1.0;
      }
      const double r = sqrt(p);
      S[j * kLeafPitch + j] = r;
      invd[j] = 1.0 / r;
    }
    __syncthreads();
    const double rinv = invd[j];
    for (int i = j + 1 + tid; i < s; i += kLeafThreads) S[i * kLeafPitch + j] *= rinv;
    __syncthreads();
    for (int i = j + 1 + ti; i < s; i += 32) {
      const double lij = S[i * kLeafPitch + j];
      for (int k = j + 1 + tk; k <= i; k += 32) S[i * kLeafPitch + k] -= lij * S[k * kLeafPitch + j];
    }
    // the next pivot is written by this loop; the barrier at the top of the
    // next iteration (after thread 0's section) is not enough for thread 0 itself
    __syncthreads();
  }

  // inverse by forward substitution, eight threads per column c:
  //   x_c[c] = 1/L_cc,   x_c[i] = -(sum_{k=c}^{i-1} L_ik x_c[k]) / L_ii
  // x_c[k] (k > c) is kept at S[c][k]; columns are independent of each other.
  const int c = tid >> 3, q = tid & 7;
  const bool live = c < s;
  const double xcc = live ? invd[c] : 0.0;
  for (int i = 1; i < s; ++i) {
    double sum = 0.0;
    if (live && i > c) {
      for (int k = c + q; k < i; k += 8) {
        const double x = (k == c) ? xcc : S[c * kLeafPitch + k];
        sum += S[i * kLeafPitch + k] * x;
      }
    }
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    sum += __shfl_xor(sum, 4);
    if (live && i > c && q == 0) S[c * kLeafPitch + i] = -sum * invd[i];
    // the eight threads of a column sit in one wavefront, whose LDS accesses
    // complete in program order, so the value is visible to them on the next i
    __builtin_amdgcn_wave_barrier();
  }
  __syncthreads();

  // X(i,j), i >= j, goes to U[n-1-(o+i)][n-1-(o+j)]
  for (int e = tid; e < s * s; e += kLeafThreads) {
    const int i = e / s, j = e % s;
    if (j <= i) {
      const double x = (i == j) ? invd[i] : S[j * kLeafPitch + i];
      U[(int64_t)(n - 1 - (o + i)) * ldu + (n - 1 - (o + j))] = x;
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
__global__ __launch_bounds__(256) void node_gemm_kernel(Op op) {
  using T = DgemmTile<TM, TN>;
  extern __shared__ double smem[];
  const int i0 = blockIdx.y * T::BM, j0 = blockIdx.x * T::BN;
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

template <class Op>
void launch_node(const Op& op, int M, int N, hipStream_t st) {
  // 64 x 128 tiles once there are enough of them to fill the chip, else 64 x 64
  const int64_t big = ceil_div(M, 64) * ceil_div(N, 128);
  if (big >= 1024)
    launch_tiles<2, 4, Op>(op, M, N, st);
  else
    launch_tiles<2, 2, Op>(op, M, N, st);
}

void recurse(double* G, double* U, int ldu, int n, int o, int s, int32_t* info, hipStream_t st) {
  if (s <= kLeaf) {
    const size_t lds = (size_t)(kLeaf * kLeafPitch + kLeaf) * sizeof(double);
    leaf_kernel<<<1, kLeafThreads, lds, st>>>(G, n, o, s, U, ldu, info);
    return;
  }
  const int nb = (int)ceil_div(s, kLeaf);
  const int s1 = (nb / 2) * kLeaf;
  const int s2 = s - s1;
  Node nd{G, U, ldu, n, o, s1, s2};
  recurse(G, U, ldu, n, o, s1, info, st);
  launch_node(OpPanel{nd}, s2, s1, st);
  launch_node(OpSyrk{nd}, s2, s2, st);
  recurse(G, U, ldu, n, o + s1, s2, info, st);
  launch_node(OpT{nd}, s2, s1, st);
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
    const int lds = (kLeaf * kLeafPitch + kLeaf) * (int)sizeof(double);
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(leaf_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
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
