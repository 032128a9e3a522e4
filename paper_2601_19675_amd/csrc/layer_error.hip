// Relative layer error  sqrt( tr(D H D^T) / tr(W H W^T) ),  D = W - Wq.
//
// H is symmetric and only its upper triangle is stored, so each quadratic form
// is evaluated as  sum_ij A_ij * (A Hu)_ij  with
//     Hu(k,j) = 2 H(k,j) for k < j,  H(k,k) for k == j,  0 for k > j,
// which reads every stored entry once in its coalesced direction and halves the
// work of the float64 MFMA GEMM (the k range of a column tile stops at its last
// column).  Each workgroup reduces its 128 x 128 tile to one number; a final
// single-workgroup kernel adds the tile sums in index order.
#include "dgemm.h"

namespace ptq {
namespace {

constexpr int TM = 2, TN = 4;  // 64 x 128 tile: two workgroups (8 waves) per CU keep the f64 matrix pipe fuller
using Tile = DgemmTile<TM, TN>;

struct ErrArgs {
  const double* A2;  // [2][m][n]: D = W - Wq, then W, both widened to float64
  int m, n;
  const double* H;
  int ldh;
  double* partial;  // [2][tiles]
};

// D = W - Wq and W itself as float64, so that the GEMM streams plain doubles.
template <int DT>
__global__ __launch_bounds__(256) void widen_kernel(const void* __restrict__ W, int64_t ldw,
                                                    const double* __restrict__ Wq, int m, int n,
                                                    double* __restrict__ A2) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * n) return;
  const int i = (int)(e / n), k = (int)(e - (int64_t)i * n);
  const double w = load_as_f64<DT>(W, (int64_t)i * ldw + k);
  A2[e] = w - Wq[e];
  A2[(int64_t)m * n + e] = w;
}

__global__ __launch_bounds__(256, 3) void quad_form_kernel(ErrArgs a) {   // three workgroups per CU fit in LDS
  extern __shared__ double smem[];
  __shared__ double red[256];
  // column tiles have k ranges proportional to their index: the widest are dispatched
  // first (blockIdx.y is the slow grid index), the two quadratic forms share blockIdx.x
  const int nrt = gridDim.x >> 1;
  const int z = blockIdx.x / nrt;
  const int rt = blockIdx.x - z * nrt;
  const int ct = gridDim.y - 1 - blockIdx.y;
  const int i0 = rt * Tile::BM, j0 = ct * Tile::BN;
  const int j1 = min(j0 + Tile::BN, a.n);
  const int i1 = min(i0 + Tile::BM, a.m);
  const double* Az = a.A2 + (int64_t)z * a.m * a.n;
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  dgemm_mainloop<TM, TN, true, false>(
      acc, DView{Az + (int64_t)i0 * a.n, a.n, 1}, DgemmIdentity{},
      // H below the diagonal is read (it is valid memory) and discarded
      DView{a.H + j0, 1, a.ldh},
      [&](double h, int k, int j) { return k == j0 + j ? h : (k < j0 + j ? 2.0 * h : 0.0); },
      i1 - i0, j1 - j0, 0, j1, smem);
  double s = 0.0;
  dgemm_foreach(acc, [&](int i, int j, double v) {
    const bool ok = (i0 + i < a.m) & (j0 + j < a.n);
    const double d = Az[ok ? (int64_t)(i0 + i) * a.n + j0 + j : 0];
    s = fma(v, ok ? d : 0.0, s);
  });
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    a.partial[((int64_t)z * nrt + rt) * gridDim.y + ct] = red[0];
}

__global__ __launch_bounds__(256) void finish_kernel(const double* __restrict__ partial, int tiles,
                                                     double* out) {
  __shared__ double red[2][256];
  for (int z = 0; z < 2; ++z) {
    double s = 0.0;
    for (int i = threadIdx.x; i < tiles; i += 256) s += partial[(int64_t)z * tiles + i];
    red[z][threadIdx.x] = s;
  }
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) {
      red[0][threadIdx.x] += red[0][threadIdx.x + w];
      red[1][threadIdx.x] += red[1][threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double num = red[0][0], den = red[1][0];
    out[0] = sqrt(num / den);
    out[1] = num;
    out[2] = den;
  }
}

}  // namespace

static size_t partial_bytes(int64_t m, int64_t n) {
  const size_t tiles = (size_t)ceil_div(m, Tile::BM) * (size_t)ceil_div(n, Tile::BN);
  return align_up(2 * tiles * sizeof(double), 256);
}

size_t layer_error_workspace_bytes(int64_t m, int64_t n) {
  return partial_bytes(m, n) + align_up(2 * (size_t)m * (size_t)n * sizeof(double), 256);
}

ptq_status layer_error_launch(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                              int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                              size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < layer_error_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  double* partial = static_cast<double*>(ws);
  double* A2 = reinterpret_cast<double*>(static_cast<char*>(ws) + partial_bytes(m, n));
  const unsigned wg = (unsigned)ceil_div(m * n, 256);
  switch (wdt) {
    case PTQ_F32: widen_kernel<PTQ_F32><<<wg, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, A2); break;
    case PTQ_BF16: widen_kernel<PTQ_BF16><<<wg, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, A2); break;
    case PTQ_F64: widen_kernel<PTQ_F64><<<wg, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, A2); break;
    default: return PTQ_ERR_DTYPE;
  }
  ErrArgs a{A2, (int)m, (int)n, H, (int)ldh, partial};
  dim3 g(2 * (unsigned)ceil_div(m, Tile::BM), (unsigned)ceil_div(n, Tile::BN));
  const int tiles = (int)(g.x / 2 * g.y);
  constexpr int lds = Tile::kSmemDoubles * (int)sizeof(double);
  if (!lds_opt_in<quad_form_kernel>(lds)) return PTQ_ERR_HIP;
  quad_form_kernel<<<g, 256, lds, st>>>(a);
  finish_kernel<<<1, 256, 0, st>>>(partial, tiles, out);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
