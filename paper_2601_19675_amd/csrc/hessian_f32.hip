// Proxy-Hessian accumulation for float32 activations:  partial tiles of  X^T X  on the float64 matrix
// cores (Sec. 2, Eq. 1; the float32 case of Algorithm 1's Hessian stage).
//
// A float32 widened to float64 is exact and so is the product of two of them, so with
// v_mfma_f64_16x16x4 the only roundings are those of the float64 sums: the result has the accuracy
// of a float64 Gram matrix, at the rate of the matrix cores instead of the vector unit's.
//
// A workgroup of four waves (2 x 2) owns a (32 WT) x (32 WT) tile of channels x channels and a chunk
// of tokens; a wave owns WT x WT tiles of the 16 x 16 x 4 instruction.  X lies [token][channel], and
// that is also what the instruction wants: lane l of an operand holds (channel l % 16, token l / 16)
// -- sixteen neighbouring channels of one token -- so a stage of 16 tokens goes into LDS as it lies in
// memory (float32, widened after the LDS read), with a row pitch that puts the four token rows of a
// fragment on different banks.  Two LDS buffers, one barrier per stage, the next stage's global loads
// in flight during the MFMAs.  Partial tiles are float64; the reduction kernel of hessian.hip adds
// them into H in a fixed order.
//
// Compiled with the accumulators of the float64 MFMA in ordinary VGPRs (the bf16 kernels of hessian.hip
// need the accumulation registers instead, hence a file of its own).
#include "common.h"

namespace ptq {
namespace {

constexpr int kKT = 16;  // tokens per stage

template <int WT>
__global__ __launch_bounds__(256) void hessian_f32_mfma_kernel(const float* __restrict__ X, int64_t ldx, int64_t t,
                                                               int n, int64_t tok0, int chunk, int ntb,
                                                               double* __restrict__ partial) {
  constexpr int TILE = 32 * WT;
  constexpr int PITCH = TILE + 16;        // floats: consecutive token rows are 16 banks apart
  constexpr int EPT = kKT * TILE / 256;   // elements per thread, stage and operand
  __shared__ float As[2][kKT * PITCH];
  __shared__ float Bs[2][kKT * PITCH];

  // upper-triangular tile list, row by row: row I holds ntb - I tiles
  int I = 0, J = (int)blockIdx.x;
  while (J >= ntb - I) {
    J -= ntb - I;
    ++I;
  }
  J += I;
  const bool diag = (I == J);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave >> 1, wj = wave & 1;
  const int64_t kbeg = tok0 + (int64_t)blockIdx.y * chunk;
  const int64_t kend = (kbeg + chunk < t) ? kbeg + chunk : t;

  f64x4 acc[WT][WT];
#pragma unroll
  for (int a = 0; a < WT; ++a)
#pragma unroll
    for (int b = 0; b < WT; ++b) acc[a][b] = f64x4{0.0, 0.0, 0.0, 0.0};

  // global -> registers -> LDS: element e = tid + 256 p of a stage is (token e / TILE, channel e % TILE):
  // neighbouring threads take neighbouring channels.  Tokens past the chunk and channels past n read as 0.
  float ra[EPT], rb[EPT];
  auto fetch = [&](int64_t k0) {
#pragma unroll
    for (int p = 0; p < EPT; ++p) {
      const int e = tid + 256 * p;
      const int kk = e / TILE, c = e % TILE;
      const int64_t k = k0 + kk;
      const int ca = I * TILE + c, cb = J * TILE + c;
      ra[p] = (k < kend && ca < n) ? X[k * ldx + ca] : 0.f;
      if (!diag) rb[p] = (k < kend && cb < n) ? X[k * ldx + cb] : 0.f;
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int p = 0; p < EPT; ++p) {
      const int e = tid + 256 * p;
      const int kk = e / TILE, c = e % TILE;
      As[buf][kk * PITCH + c] = ra[p];
      if (!diag) Bs[buf][kk * PITCH + c] = rb[p];
    }
  };

  if (kbeg < kend) {
    const int fr = (lane >> 4) * PITCH + (lane & 15);  // (token l / 16, channel l % 16) inside a fragment
    fetch(kbeg);
    int buf = 0;
    for (int64_t k0 = kbeg; k0 < kend; k0 += kKT, buf ^= 1) {
      // the buffer written here was last read two stages ago; every wave has passed a barrier since
      stash(buf);
      __syncthreads();
      if (k0 + kKT < kend) fetch(k0 + kKT);
      const float* At = As[buf];
      const float* Bt = diag ? As[buf] : Bs[buf];
#pragma unroll
      for (int ks = 0; ks < kKT / 4; ++ks) {
        double fa[WT], fb[WT];
#pragma unroll
        for (int a = 0; a < WT; ++a) fa[a] = (double)At[ks * 4 * PITCH + fr + (wi * WT + a) * 16];
#pragma unroll
        for (int b = 0; b < WT; ++b) fb[b] = (double)Bt[ks * 4 * PITCH + fr + (wj * WT + b) * 16];
#pragma unroll
        for (int a = 0; a < WT; ++a)
#pragma unroll
          for (int b = 0; b < WT; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(fa[a], fb[b], acc[a][b], 0, 0, 0);
      }
    }
  }

  // result layout of the float64 instruction: lane l, register r holds (row 4 r + l / 16, column l % 16)
  double* out = partial + ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (TILE * TILE);
#pragma unroll
  for (int a = 0; a < WT; ++a)
#pragma unroll
    for (int b = 0; b < WT; ++b)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        out[((wi * WT + a) * 16 + 4 * r + (lane >> 4)) * TILE + (wj * WT + b) * 16 + (lane & 15)] = acc[a][b][r];
}

}  // namespace

// Partial tiles of `tile` x `tile` (64 or 128) doubles for grid.x tiles and grid.y chunks of `chunk` tokens.
bool hessian_f32_partials_launch(const float* X, int64_t ldx, int64_t t, int n, int64_t tok0, int chunk, int ntb,
                                 int tile, dim3 grid, double* partial, hipStream_t st) {
  if (tile == 128)
    hessian_f32_mfma_kernel<4><<<grid, 256, 0, st>>>(X, ldx, t, n, tok0, chunk, ntb, partial);
  else if (tile == 64)
    hessian_f32_mfma_kernel<2><<<grid, 256, 0, st>>>(X, ldx, t, n, tok0, chunk, ntb, partial);
  else
    return false;
  return true;
}

}  // namespace ptq
