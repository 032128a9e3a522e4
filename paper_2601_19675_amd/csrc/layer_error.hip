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

constexpr int TM = 4, TN = 4;
using Tile = DgemmTile<TM, TN>;

struct ErrArgs {
  const void* W;
  int64_t ldw;
  const double* Wq;
  int m, n;
  const double* H;
  int64_t ldh;
  double* partial;  // [2][tiles]
};

template <int DT>
__global__ __launch_bounds__(256) void quad_form_kernel(ErrArgs a) {
  __shared__ double smem[Tile::kSmemDoubles];
  __shared__ double red[256];
  const int z = blockIdx.z;
  const int i0 = blockIdx.y * Tile::BM, j0 = blockIdx.x * Tile::BN;
  const int j1 = min(j0 + Tile::BN, a.n);
  const int i1 = min(i0 + Tile::BM, a.m);
  // element of D (z == 0) or W (z == 1); indices always inside the matrix
  auto elem = [&](int i, int k) -> double {
    const double w = load_as_f64<DT>(a.W, (int64_t)i * a.ldw + k);
    const double q = a.Wq[(int64_t)i * a.n + k];
    return z == 0 ? w - q : w;
  };
  f64x4 acc[TM][TN];
  dgemm_zero(acc);
  dgemm_mainloop<TM, TN, true, false>(
      acc, [&](int i, int k) { return elem(i0 + i, k); },
      [&](int k, int j) {
        const int gj = j0 + j;
        const double h = a.H[(int64_t)k * a.ldh + gj];  // below the diagonal: read, then discarded
        return k == gj ? h : (k < gj ? 2.0 * h : 0.0);
      },
      i1 - i0, j1 - j0, 0, j1, smem);
  double s = 0.0;
  dgemm_foreach(acc, [&](int i, int j, double v) {
    const bool ok = (i0 + i < a.m) & (j0 + j < a.n);
    const double d = elem(ok ? i0 + i : i0, ok ? j0 + j : j0);
    s = fma(v, ok ? d : 0.0, s);
  });
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    a.partial[(int64_t)z * gridDim.x * gridDim.y + blockIdx.y * gridDim.x + blockIdx.x] = red[0];
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

size_t layer_error_workspace_bytes(int64_t m, int64_t n) {
  const size_t tiles = (size_t)ceil_div(m, Tile::BM) * (size_t)ceil_div(n, Tile::BN);
  return align_up(2 * tiles * sizeof(double), 256);
}

ptq_status layer_error_launch(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                              int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                              size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < layer_error_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  ErrArgs a{W, ldw, Wq, (int)m, (int)n, H, ldh, static_cast<double*>(ws)};
  dim3 g((unsigned)ceil_div(n, Tile::BN), (unsigned)ceil_div(m, Tile::BM), 2);
  const int tiles = (int)(g.x * g.y);
  switch (wdt) {
    case PTQ_F32: quad_form_kernel<PTQ_F32><<<g, 256, 0, st>>>(a); break;
    case PTQ_BF16: quad_form_kernel<PTQ_BF16><<<g, 256, 0, st>>>(a); break;
    case PTQ_F64: quad_form_kernel<PTQ_F64><<<g, 256, 0, st>>>(a); break;
    default: return PTQ_ERR_DTYPE;
  }
  finish_kernel<<<1, 256, 0, st>>>(a.partial, tiles, out);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
