// Relative layer error  sqrt( tr(D H D^T) / tr(W H W^T) ),  D = W - Wq.
//
// H is symmetric and only its upper triangle is stored, so each quadratic form
// is evaluated as  sum_ij A_ij * (A Hu)_ij  with
//     Hu(k,j) = 2 H(k,j) for k < j,  H(k,k) for k == j,  0 for k > j,
// which reads every stored entry once in its coalesced direction and halves the
// work of the float64 MFMA GEMM (the k range of a column tile stops at its last
// column).  Each workgroup reduces its tile to one number; a final
// single-workgroup kernel adds the tile sums in index order.
//
// Two forms of the same sum.  Weights stored in float64 take the float64 MFMA GEMM.  Weights
// stored in float32 or bfloat16 take the float32 one: D, W and Hu are rounded to float32 once
// (W in bfloat16 is exact), products and the running sums over k are float32 on the matrix
// cores, and everything from the tile's sum_ij A_ij T_ij on is float64.  The roundings are
// unbiased and independent, so they average out over the m n terms of the trace: measured
// against the float64 definition the two traces differ by a few parts in 10^8.
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

// D = W - Wq next to W itself, both dense, so that the GEMM streams two plain matrices.
__global__ __launch_bounds__(256) void widen_kernel(const double* __restrict__ W, int64_t ldw,
                                                    const double* __restrict__ Wq, int m, int n,
                                                    double* __restrict__ A2) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * n) return;
  const int i = (int)(e / n), k = (int)(e - (int64_t)i * n);
  const double w = W[(int64_t)i * ldw + k];
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

// ---------------------------------------------------------------- float32 matrix-core form
constexpr int kT = 128;          // tile edge: four waves, 64 x 64 each (2 x 2 tiles of the 32 x 32 x 2 MFMA)
constexpr int kBK = 16;          // k-tile
constexpr int kPitch = kT + 32;  // LDS pitch: the two k rows of a fragment read fall on the two bank halves

struct Err32Args {
  const float* A32;  // [2][mp][np]: D = W - Wq, then W; zero outside m x n
  const float* Hu;   // [np][np]: Hu; zero below the diagonal and outside n x n
  int mp, np;        // m, n rounded up to the tile edge
  double* partial;   // [2][tiles]
};

template <int DT>
__global__ __launch_bounds__(256) void narrow_kernel(const void* __restrict__ W, int64_t ldw,
                                                     const double* __restrict__ Wq, int m, int n, int mp, int np,
                                                     float* __restrict__ A32) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;   // four consecutive k
  if (q >= (int64_t)mp * np / 4) return;
  const int i = (int)(q / (np / 4)), k0 = (int)(q - (int64_t)i * (np / 4)) * 4;
  float d[4], w[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const bool ok = i < m && k0 + c < n;
    const double wv = ok ? load_as_f64<DT>(W, (int64_t)i * ldw + k0 + c) : 0.0;
    const double qv = ok ? Wq[(int64_t)i * n + k0 + c] : 0.0;
    d[c] = (float)(wv - qv);
    w[c] = (float)wv;
  }
  float* o = A32 + (int64_t)i * np + k0;
  *reinterpret_cast<float4*>(o) = float4{d[0], d[1], d[2], d[3]};
  *reinterpret_cast<float4*>(o + (int64_t)mp * np) = float4{w[0], w[1], w[2], w[3]};
}

__global__ __launch_bounds__(256) void hu_kernel(const double* __restrict__ H, int64_t ldh, int n, int np,
                                                 float* __restrict__ Hu) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;   // four consecutive j
  if (q >= (int64_t)np * np / 4) return;
  const int k = (int)(q / (np / 4)), j0 = (int)(q - (int64_t)k * (np / 4)) * 4;
  float v[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int j = j0 + c;
    const bool ok = k < n && j < n && k <= j;
    const double h = ok ? H[(int64_t)k * ldh + j] : 0.0;
    v[c] = (float)(k == j ? h : 2.0 * h);
  }
  *reinterpret_cast<float4*>(Hu + (int64_t)k * np + j0) = float4{v[0], v[1], v[2], v[3]};
}

__global__ __launch_bounds__(256, 2) void quad_form32_kernel(Err32Args a) {
  __shared__ float As[2][kBK][kPitch];   // [stage][k][i]
  __shared__ float Bs[2][kBK][kPitch];   // [stage][k][j]
  __shared__ double red[4];
  // column tiles have k ranges proportional to their index: the widest are dispatched first
  // (blockIdx.y is the slow grid index), the two quadratic forms share blockIdx.x
  const int nrt = gridDim.x >> 1;
  const int z = blockIdx.x / nrt;
  const int rt = blockIdx.x - z * nrt;
  const int ct = gridDim.y - 1 - blockIdx.y;
  const int i0 = rt * kT, j0 = ct * kT;
  const int kend = j0 + kT;   // below it Hu is zero; a multiple of the k-tile
  const float* __restrict__ A = a.A32 + ((int64_t)z * a.mp + i0) * a.np;
  const float* __restrict__ B = a.Hu + j0;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // global -> registers -> LDS: a thread brings 8 consecutive k of one row of A and 8 consecutive j of one row of Hu
  const int ar = tid >> 1, ak = (tid & 1) * 8;
  const int bk = tid >> 4, bj = (tid & 15) * 8;
  const float* ap = A + (int64_t)ar * a.np + ak;
  const float* bp = B + (int64_t)bk * a.np + bj;
  float4 ra0, ra1, rb0, rb1;
  auto fetch = [&](int k0) {
    ra0 = *reinterpret_cast<const float4*>(ap + k0);
    ra1 = *reinterpret_cast<const float4*>(ap + k0 + 4);
    rb0 = *reinterpret_cast<const float4*>(bp + (int64_t)k0 * a.np);
    rb1 = *reinterpret_cast<const float4*>(bp + (int64_t)k0 * a.np + 4);
  };
  auto stash = [&](int s) {
    As[s][ak + 0][ar] = ra0.x; As[s][ak + 1][ar] = ra0.y; As[s][ak + 2][ar] = ra0.z; As[s][ak + 3][ar] = ra0.w;
    As[s][ak + 4][ar] = ra1.x; As[s][ak + 5][ar] = ra1.y; As[s][ak + 6][ar] = ra1.z; As[s][ak + 7][ar] = ra1.w;
    *reinterpret_cast<float4*>(&Bs[s][bk][bj]) = rb0;
    *reinterpret_cast<float4*>(&Bs[s][bk][bj + 4]) = rb1;
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0.f;

  fetch(0);
  stash(0);
  if (kBK < kend) fetch(kBK);
  __syncthreads();
  int cur = 0;
  for (int k0 = 0; k0 < kend; k0 += kBK) {
    // next k-tile: registers -> the other stage; the one after: issue its loads
    if (k0 + kBK < kend) stash(cur ^ 1);
    if (k0 + 2 * kBK < kend) fetch(k0 + 2 * kBK);
    // operand fragments: lane l holds A(i = l % 32, k = l / 32) and B(k = l / 32, j = l % 32)
#pragma unroll
    for (int ks = 0; ks < kBK / 2; ++ks) {
      const int kr = 2 * ks + (lane >> 5);
      float av[2], bv[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        av[t] = As[cur][kr][wm * 64 + t * 32 + (lane & 31)];
        bv[t] = Bs[cur][kr][wn * 64 + t * 32 + (lane & 31)];
      }
#pragma unroll
      for (int tm = 0; tm < 2; ++tm)
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
          acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[tm], bv[tn], acc[tm][tn], 0, 0, 0);
    }
    __syncthreads();   // stage cur free for the tile after next, stage cur ^ 1 complete
    cur ^= 1;
  }

  // sum_ij A_ij T_ij of the tile in float64; accumulator r of a lane is row (r / 4) * 8 + (lane / 32) * 4 + r % 4,
  // column lane % 32 of its 32 x 32 tile; rows and columns beyond m x n hold zeros
  double s = 0.0;
#pragma unroll
  for (int tm = 0; tm < 2; ++tm)
#pragma unroll
    for (int tn = 0; tn < 2; ++tn)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = wm * 64 + tm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int j = wn * 64 + tn * 32 + (lane & 31);
        s = fma((double)acc[tm][tn][r], (double)A[(int64_t)i * a.np + j0 + j], s);
      }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (tid == 0) a.partial[((int64_t)z * nrt + rt) * gridDim.y + ct] = (red[0] + red[1]) + (red[2] + red[3]);
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

static size_t bytes_f64_form(int64_t m, int64_t n) {
  return partial_bytes(m, n) + align_up(2 * (size_t)m * (size_t)n * sizeof(double), 256);
}

static size_t partial32_bytes(int64_t mp, int64_t np) {
  return align_up(2 * (size_t)(mp / kT) * (size_t)(np / kT) * sizeof(double), 256);
}

static size_t bytes_f32_form(int64_t m, int64_t n) {
  const int64_t mp = ceil_div(m, kT) * kT, np = ceil_div(n, kT) * kT;
  return partial32_bytes(mp, np) + align_up(2 * (size_t)mp * (size_t)np * sizeof(float), 256) +
         align_up((size_t)np * (size_t)np * sizeof(float), 256);
}

// the caller asks before it says which storage type W has: enough for either form
size_t layer_error_workspace_bytes(int64_t m, int64_t n) {
  const size_t a = bytes_f64_form(m, n), b = bytes_f32_form(m, n);
  return a > b ? a : b;
}

static ptq_status launch_f32_form(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m, int64_t n,
                                  const double* H, int64_t ldh, double* out, void* ws, hipStream_t st) {
  const int64_t mp = ceil_div(m, kT) * kT, np = ceil_div(n, kT) * kT;
  double* partial = static_cast<double*>(ws);
  float* A32 = reinterpret_cast<float*>(static_cast<char*>(ws) + partial32_bytes(mp, np));
  float* Hu = reinterpret_cast<float*>(reinterpret_cast<char*>(A32) +
                                       align_up(2 * (size_t)mp * (size_t)np * sizeof(float), 256));
  const unsigned ga = (unsigned)ceil_div(mp * np / 4, 256), gh = (unsigned)ceil_div(np * np / 4, 256);
  if (wdt == PTQ_F32)
    narrow_kernel<PTQ_F32><<<ga, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, (int)mp, (int)np, A32);
  else
    narrow_kernel<PTQ_BF16><<<ga, 256, 0, st>>>(W, ldw, Wq, (int)m, (int)n, (int)mp, (int)np, A32);
  hu_kernel<<<gh, 256, 0, st>>>(H, ldh, (int)n, (int)np, Hu);
  Err32Args a{A32, Hu, (int)mp, (int)np, partial};
  dim3 g(2 * (unsigned)(mp / kT), (unsigned)(np / kT));
  quad_form32_kernel<<<g, 256, 0, st>>>(a);
  finish_kernel<<<1, 256, 0, st>>>(partial, (int)(g.x / 2 * g.y), out);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status layer_error_launch(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                              int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                              size_t ws_bytes, hipStream_t st) {
  if (ws_bytes < layer_error_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  if (wdt == PTQ_F32 || wdt == PTQ_BF16) return launch_f32_form(W, wdt, ldw, Wq, m, n, H, ldh, out, ws, st);
  if (wdt != PTQ_F64) return PTQ_ERR_DTYPE;
  double* partial = static_cast<double*>(ws);
  double* A2 = reinterpret_cast<double*>(static_cast<char*>(ws) + partial_bytes(m, n));
  const unsigned wg = (unsigned)ceil_div(m * n, 256);
  widen_kernel<<<wg, 256, 0, st>>>(static_cast<const double*>(W), ldw, Wq, (int)m, (int)n, A2);
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
