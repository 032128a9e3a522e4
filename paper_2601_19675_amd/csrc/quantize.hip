// Blocked column-by-column quantization with error compensation.
//
// Rows of W are independent given the factor U, so a workgroup owns 16 rows
// (one MFMA M-tile) and nothing is exchanged between workgroups.  The lazy
// update is applied "left-looking": when the column loop arrives at block
// [i1, i2), the block's current values are
//
//     S = W[:, i1:i2] - E[:, 0:i1] * U[0:i1, i1:i2]            (float64 MFMA)
//
// with E the errors e_j of all earlier columns (kept transposed, [n][rows], in
// the workspace).  That is the same sum the right-looking rank-B updates would
// have accumulated, but it reads E once and writes nothing but the block.
// Inside the block the same scheme repeats with 16-column mini-blocks: one lane
// per row walks 16 columns in registers (the only truly serial part), then the
// 16 new errors are pushed onto the rest of the block with four MFMAs per
// 16-column tile.
#include "common.h"

namespace ptq {
namespace {

constexpr int kRows = 16;       // rows per workgroup
constexpr int kMaxTiles = 16;   // block <= 256 columns
constexpr int kThreads = 256;

__global__ void inv_diag_kernel(const double* __restrict__ U, int64_t ldu, int n, double* invd) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) invd[j] = 1.0 / U[(int64_t)j * ldu + j];
}

struct QuantArgs {
  const void* W;
  int64_t ldw;
  int m, n, mpad;
  const double* U;
  int64_t ldu;
  const uint8_t* dead;
  const double* invd;
  double* errT;  // [n][mpad]
  int bits, group;
  int i1, bw;    // block start, block width (multiple of 16)
  uint8_t* codes;
  float* scales;
  uint8_t* zeros;
  double* Wq;
  double* row_err2;
};

template <int DT>
__global__ __launch_bounds__(kThreads) void quant_block_kernel(QuantArgs a) {
  extern __shared__ double lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int row0 = blockIdx.x * kRows;
  const int nt = a.bw >> 4;
  const int sp = a.bw + 1;  // pitch of the state tile

  // LDS carve-up: partial sums of the four waves (reused as the state tile),
  // the mini-block errors, group min / max, and the code tile.
  double* P = lds;                                  // [4][16][bw]
  double* S = lds;                                  // [16][bw + 1]   (aliases P)
  double* Em = lds + 4 * kRows * a.bw;              // [16 k][16 rows]
  double* gmin = Em + 256;                          // [16]
  double* gmax = gmin + 16;                         // [16]
  uint8_t* Ct = reinterpret_cast<uint8_t*>(gmax + 16);  // [16][bw]

  // ---- phase 1: acc = E[rows, 0:i1] * U[0:i1, block], k split over the waves
  f64x4 acc[kMaxTiles];
#pragma unroll
  for (int t = 0; t < kMaxTiles; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
  {
    const int kl = lane >> 4, cl = lane & 15;
    const double* ep = a.errT + (int64_t)(4 * wave + kl) * a.mpad + row0 + cl;
    const double* up = a.U + (int64_t)(4 * wave + kl) * a.ldu + a.i1 + cl;
    for (int k0 = 4 * wave; k0 < a.i1; k0 += 16) {
      const double av = *ep;
      double bv[kMaxTiles];
#pragma unroll
      for (int t = 0; t < kMaxTiles; ++t) bv[t] = (t < nt) ? up[16 * t] : 0.0;
#pragma unroll
      for (int t = 0; t < kMaxTiles; ++t)
        if (t < nt) acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv[t], acc[t], 0, 0, 0);
      ep += (int64_t)16 * a.mpad;
      up += (int64_t)16 * a.ldu;
    }
  }
#pragma unroll
  for (int t = 0; t < kMaxTiles; ++t)
    if (t < nt) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        P[(wave * kRows + 4 * r + (lane >> 4)) * a.bw + 16 * t + (lane & 15)] = acc[t][r];
    }
  __syncthreads();

  // ---- state tile S = W - (p0 + p1 + p2 + p3), dead channels read as zero
  {
    double sv[kMaxTiles];
#pragma unroll
    for (int p = 0; p < kMaxTiles; ++p) {
      const int e = tid + kThreads * p;
      sv[p] = 0.0;
      if (e < kRows * a.bw) {
        const int r = e / a.bw, c = e - r * a.bw;
        double w = 0.0;
        if (row0 + r < a.m && !(a.dead && a.dead[a.i1 + c]))
          w = load_as_f64<DT>(a.W, (int64_t)(row0 + r) * a.ldw + a.i1 + c);
        const double s01 = P[(0 * kRows + r) * a.bw + c] + P[(1 * kRows + r) * a.bw + c];
        const double s23 = P[(2 * kRows + r) * a.bw + c] + P[(3 * kRows + r) * a.bw + c];
        sv[p] = w - (s01 + s23);
      }
    }
    __syncthreads();
#pragma unroll
    for (int p = 0; p < kMaxTiles; ++p) {
      const int e = tid + kThreads * p;
      if (e < kRows * a.bw) {
        const int r = e / a.bw, c = e - r * a.bw;
        S[r * sp + c] = sv[p];
      }
    }
  }
  __syncthreads();

  // ---- phase 2: 16-column mini-blocks
  const double maxq = (double)((1 << a.bits) - 1);
  const int ng = a.n / a.group;
  double scale = 1.0, rscale = 1.0, zero = 0.0, err2 = 0.0;  // live in lanes 0..15 of wave 0
  for (int mb = 0; mb < nt; ++mb) {
    const int c0 = 16 * mb;           // first column of the mini-block inside the block
    const int gcol = a.i1 + c0;       // ... and in the layer
    const bool gstart = (gcol % a.group) == 0;
    if (gstart) {
      // min / max of the group's current values: 16 lanes per row
      const int r = tid >> 4, sub = tid & 15;
      double lo = 0.0, hi = 0.0;
      for (int c = sub; c < a.group; c += 16) {
        const double v = S[r * sp + c0 + c];
        lo = fmin(lo, v);
        hi = fmax(hi, v);
      }
#pragma unroll
      for (int x = 8; x > 0; x >>= 1) {
        lo = fmin(lo, __shfl_xor(lo, x));
        hi = fmax(hi, __shfl_xor(hi, x));
      }
      if (sub == 0) {
        gmin[r] = lo;
        gmax[r] = hi;
      }
      __syncthreads();
    }
    if (tid < kRows) {
      const int r = tid;
      const bool rlive = row0 + r < a.m;
      if (gstart) {
        double lo = gmin[r], hi = gmax[r];
        if (lo == hi) {
          lo = -1.0;
          hi = 1.0;
        }
        const float sf = (float)((hi - lo) / maxq);
        scale = (double)sf;
        rscale = 1.0 / scale;
        zero = rint(-lo / scale);
        if (rlive) {
          a.scales[(int64_t)(row0 + r) * ng + gcol / a.group] = sf;
          a.zeros[(int64_t)(row0 + r) * ng + gcol / a.group] = (uint8_t)zero;
        }
      }
      double w[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = S[r * sp + c0 + j];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        // x = w / scale, correctly rounded from the reciprocal (one Newton step
        // on the quotient), so that exact ties round as a true division would
        const double q0 = w[j] * rscale;
        const double rem = fma(-q0, scale, w[j]);
        const double x = fma(rem, rscale, q0);
        const double code = fmin(fmax(rint(x) + zero, 0.0), maxq);
        const double q = scale * (code - zero);
        const double e = (w[j] - q) * a.invd[gcol + j];
        const double* urow = a.U + (int64_t)(gcol + j) * a.ldu + gcol;
#pragma unroll
        for (int k = j + 1; k < 16; ++k) w[k] = fma(-e, urow[k], w[k]);
        err2 = fma(e, e, err2);
        Ct[r * a.bw + c0 + j] = (uint8_t)code;
        Em[j * kRows + r] = e;
        a.errT[(int64_t)(gcol + j) * a.mpad + row0 + r] = e;
        if (a.Wq && rlive) a.Wq[(int64_t)(row0 + r) * a.n + gcol + j] = q;
      }
    }
    __syncthreads();
    // push the 16 new errors onto the later tiles of the block
    for (int t = mb + 1 + wave; t < nt; t += 4) {
      f64x4 d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int kk = 0; kk < 16; kk += 4) {
        const int k = kk + (lane >> 4);
        const double av = Em[k * kRows + (lane & 15)];
        const double bv = a.U[(int64_t)(gcol + k) * a.ldu + a.i1 + 16 * t + (lane & 15)];
        d = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, d, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r) S[(4 * r + (lane >> 4)) * sp + 16 * t + (lane & 15)] -= d[r];
    }
    __syncthreads();
  }

  // ---- outputs of the block
  for (int e = tid; e < kRows * a.bw; e += kThreads) {
    const int r = e / a.bw, c = e - r * a.bw;
    if (row0 + r < a.m) a.codes[(int64_t)(row0 + r) * a.n + a.i1 + c] = Ct[r * a.bw + c];
  }
  if (a.row_err2 && tid < kRows && row0 + tid < a.m) {
    if (a.i1 == 0)
      a.row_err2[row0 + tid] = err2;
    else
      a.row_err2[row0 + tid] += err2;
  }
}

size_t block_lds_bytes(int bw) {
  return (size_t)(4 * kRows * bw + 256 + 32) * sizeof(double) + (size_t)kRows * bw;
}

template <int DT>
ptq_status run_blocks(QuantArgs a, int block, hipStream_t st) {
  const size_t max_lds = block_lds_bytes(block);
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(quant_block_kernel<DT>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)max_lds) != hipSuccess)
    return PTQ_ERR_HIP;
  for (int i1 = 0; i1 < a.n; i1 += block) {
    a.i1 = i1;
    a.bw = (a.n - i1 < block) ? a.n - i1 : block;
    quant_block_kernel<DT><<<a.mpad / kRows, kThreads, block_lds_bytes(a.bw), st>>>(a);
  }
  return PTQ_OK;
}

}  // namespace

size_t quantize_workspace_bytes(int64_t m, int64_t n) {
  const int64_t mpad = ceil_div(m, kRows) * kRows;
  return align_up((size_t)n * (size_t)mpad * sizeof(double), 256) + align_up((size_t)n * sizeof(double), 256);
}

ptq_status quantize_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                           const double* U, int64_t ldu, const uint8_t* dead_mask, int bits, int group,
                           int block, uint8_t* codes, float* scales, uint8_t* zeros, double* Wq,
                           double* row_err2, void* ws, size_t ws_bytes, hipStream_t st) {
  if (m == 0 || n == 0) return PTQ_OK;
  if (ws_bytes < quantize_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  // a group wider than the block makes the grid depend on columns beyond the
  // block: run with the block widened to the group (the block size only
  // changes the order of summation)
  if (group > block) block = group;
  QuantArgs a;
  a.W = W;
  a.ldw = ldw;
  a.m = (int)m;
  a.n = (int)n;
  a.mpad = (int)(ceil_div(m, kRows) * kRows);
  a.U = U;
  a.ldu = ldu;
  a.dead = dead_mask;
  a.errT = static_cast<double*>(ws);
  a.invd = reinterpret_cast<double*>(static_cast<char*>(ws) +
                                     align_up((size_t)n * (size_t)a.mpad * sizeof(double), 256));
  a.bits = bits;
  a.group = group;
  a.i1 = 0;
  a.bw = 0;
  a.codes = codes;
  a.scales = scales;
  a.zeros = zeros;
  a.Wq = Wq;
  a.row_err2 = row_err2;
  inv_diag_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(U, ldu, (int)n, const_cast<double*>(a.invd));
  PTQ_HIP_CHECK_LAUNCH();
  ptq_status rc;
  switch (wdt) {
    case PTQ_F32: rc = run_blocks<PTQ_F32>(a, block, st); break;
    case PTQ_BF16: rc = run_blocks<PTQ_BF16>(a, block, st); break;
    case PTQ_F64: rc = run_blocks<PTQ_F64>(a, block, st); break;
    default: return PTQ_ERR_DTYPE;
  }
  if (rc != PTQ_OK) return rc;
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
