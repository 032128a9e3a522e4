// Vector-quantized form of the column solve: d consecutive columns of a row are assigned one of K
// codebook entries, and the error of the assignment is compensated in the later columns.
//
// Same frame as the scalar solve (quantize.hip): a workgroup owns 16 rows, the lazy update of a block
// of columns is applied left-looking in one float64 MFMA pass over the errors of all earlier columns,
// and inside the block the work goes by 16-column mini-blocks whose errors are pushed onto the later
// tiles with four MFMAs each.  What differs is the walk over a mini-block.  For a group of d columns
// starting at j, with T = U[j:j+d, j:j+d], the loss of entry c for the row's current values w is
// sum_i e_i^2 with e = (w - c) T^-1 taken by forward substitution (the errors the scalar walk would
// make column by column); the entry with the smallest loss is assigned, the lowest index among exactly
// equal ones.  Half a wave works for one row: a lane keeps K / 32 entries in registers for the whole
// walk, evaluates their losses, and the 32 lanes agree on the minimum by exchanging (loss, index)
// pairs; every lane then knows the group's errors and applies them to the later columns of the
// mini-block itself, so the eight waves walk their two rows each without a barrier between groups.
#include "common.h"

namespace ptq {
namespace {

constexpr int kRows = 16;       // rows per workgroup
constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kRowAlign = 96;   // row padding of the error matrix (the scalar solve's workspace layout)
constexpr int kSlots = 8;       // codebook entries per lane: K <= 32 * kSlots

struct VqArgs {
  const void* W;
  int64_t ldw;
  int m, n, mpad;
  const double* U;
  int64_t ldu;
  const uint8_t* dead;
  const double* invd;
  double* errT;  // [n][mpad]
  const float* codebook;  // [K][d]
  int K;
  int i1, bw;
  uint8_t* indices;  // [m][n / d]
  double* Wq;
  double* row_err2;
};

__global__ void vq_inv_diag_kernel(const double* __restrict__ U, int64_t ldu, int n, double* invd) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) invd[j] = 1.0 / U[(int64_t)j * ldu + j];
}

// (loss, index) of lane ^ MASK, by two 32-bit lane permutes per double
template <int MASK>
__device__ __forceinline__ void take_smaller(double& loss, int& idx) {
  const int lane = threadIdx.x & 63;
  const int src = (lane ^ MASK) << 2;
  const int lo = __builtin_amdgcn_ds_bpermute(src, __double2loint(loss));
  const int hi = __builtin_amdgcn_ds_bpermute(src, __double2hiint(loss));
  const int oi = __builtin_amdgcn_ds_bpermute(src, idx);
  const double ol = __hiloint2double(hi, lo);
  const bool take = (ol < loss) || (ol == loss && oi < idx);
  loss = take ? ol : loss;
  idx = take ? oi : idx;
}

template <int DT, int NT, int D>
__global__ __launch_bounds__(kThreads) void vq_block_kernel(VqArgs a) {
  extern __shared__ double lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const int row0 = blockIdx.x * kRows;
  const int nt = a.bw >> 4;
  const int sp = a.bw + 1;  // pitch of the state tile
  const double* __restrict__ U = a.U;
  const double* __restrict__ invd = a.invd;
  constexpr int G = 16 / D;  // groups per mini-block

  double* P = lds;                                  // [4][16][bw] partial sums of the lazy update
  double* S = lds;                                  // [16][bw + 1] state tile (aliases P)
  double* Em = lds + 4 * kRows * a.bw;              // [16 k][16 rows] errors of the mini-block
  double* Qm = Em + 256;                            // [16 k][17] assigned values of the mini-block
  double* Ud = Qm + 272;                            // [2][16][16] diagonal block of U
  double* Id = Ud + 512;                            // [2][16] reciprocal pivots
  uint8_t* It = reinterpret_cast<uint8_t*>(Id + 32);  // [16][bw / D] indices of the block

  // ---- phase 1: acc = E[rows, 0:i1] * U[0:i1, block], k split over the waves
  f64x4 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
  // 16-byte loads need 16-byte alignment here (plain loads): an even ldu and U itself aligned
  const bool paired = (nt % 2 == 0) && (a.ldu % 2 == 0) && ((reinterpret_cast<uintptr_t>(U) & 15) == 0);
  auto column_of = [&](int t, int cl) { return paired ? 32 * (t >> 1) + 2 * cl + (t & 1) : 16 * t + cl; };
  {
    constexpr int kDepth = (NT >= 16) ? 2 : 4;
    const int kl = lane >> 4, cl = lane & 15;
    int coff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) coff[t] = 16 * (t < nt ? t : nt - 1);
    const int niter = (a.i1 - 4 * wv + 4 * kWaves - 1) / (4 * kWaves);
    double av[kDepth], bv[kDepth][NT];
    auto mfmas = [&](int d) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[d], bv[d][t], acc[t], 0, 0, 0);
    };
    const double* ep = a.errT + (int64_t)(4 * wv + kl) * a.mpad + row0 + cl;
    const double* up = U + (int64_t)(4 * wv + kl) * a.ldu + a.i1 + cl;
    // (with a whole number of tile pairs a lane fetches two neighbouring columns of U at once, one for each
    //  tile of a pair -- tile 2p + q then works on columns 32 p + 2 cl + q; see the scalar solve for why)
    typedef double f64x2 __attribute__((ext_vector_type(2)));
    const double* up2 = U + (int64_t)(4 * wv + kl) * a.ldu + a.i1 + 2 * cl;
    auto issue = [&](int slot, int it) {
      av[slot] = ep[(int64_t)it * (4 * kWaves) * a.mpad];
      if (paired) {
        const double* u = up2 + (int64_t)it * (4 * kWaves) * a.ldu;
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
          const f64x2 two = *reinterpret_cast<const f64x2*>(u + (coff[2 * p] & ~31));
          bv[slot][2 * p] = two[0];
          bv[slot][2 * p + 1] = two[1];
        }
      } else {
        const double* u = up + (int64_t)it * (4 * kWaves) * a.ldu;
#pragma unroll
        for (int t = 0; t < NT; ++t) bv[slot][t] = u[coff[t]];
      }
    };
#pragma unroll
    for (int d = 0; d < kDepth; ++d)
      if (d < niter) issue(d, d);
    for (int it = 0; it < niter; it += kDepth) {
#pragma unroll
      for (int d = 0; d < kDepth; ++d) {
        if (it + d < niter) {
          mfmas(d);
          if (it + d + kDepth < niter) issue(d, it + d + kDepth);
        }
      }
    }
  }
  if (wave >= 4) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
      if (t < nt) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          P[((wave - 4) * kRows + 4 * r + (lane >> 4)) * a.bw + column_of(t, lane & 15)] = acc[t][r];
      }
  }
  __syncthreads();
  if (wave < 4) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
      if (t < nt) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          P[(wave * kRows + 4 * r + (lane >> 4)) * a.bw + column_of(t, lane & 15)] += acc[t][r];
      }
  }
  __syncthreads();

  // ---- state tile S = W - (p0 + p1 + p2 + p3), dead channels read as zero
  {
    constexpr int NP = (kRows * 16 * NT + kThreads - 1) / kThreads;
    double sv[NP];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
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
    for (int p = 0; p < NP; ++p) {
      const int e = tid + kThreads * p;
      if (e < kRows * a.bw) {
        const int r = e / a.bw, c = e - r * a.bw;
        S[r * sp + c] = sv[p];
      }
    }
    if (tid < 256) Ud[tid] = U[(int64_t)(a.i1 + (tid >> 4)) * a.ldu + a.i1 + (tid & 15)];
    if (tid < 16) Id[tid] = invd[a.i1 + tid];
  }
  __syncthreads();

  // ---- phase 2: 16-column mini-blocks; half a wave walks one row
  // this lane's codebook entries, k = l32 + 32 s, in registers from here on (after the lazy update, whose
  // accumulators need the room)
  const int l32 = lane & 31;
  double cb[kSlots][D];
#pragma unroll
  for (int s = 0; s < kSlots; ++s) {
    const int k = l32 + 32 * s;
#pragma unroll
    for (int i = 0; i < D; ++i) cb[s][i] = k < a.K ? (double)a.codebook[k * D + i] : 0.0;
  }
  const int r = 2 * wave + (lane >> 5);   // the row of this half-wave
  double err2 = 0.0;
  constexpr int kUpd = (NT + kWaves - 1) / kWaves;
  const int gpb = a.bw / D;               // groups per block (pitch of the index tile)
  for (int mb = 0; mb < nt; ++mb) {
    const int c0 = 16 * mb;
    const int gcol = a.i1 + c0;
    const int buf = mb & 1;
    double ud_next = 0.0, id_next = 0.0;
    if (mb + 1 < nt) {
      if (tid < 256) ud_next = U[(int64_t)(gcol + 16 + (tid >> 4)) * a.ldu + gcol + 16 + (tid & 15)];
      if (tid < 16) id_next = invd[gcol + 16 + tid];
    }
    double ub[kUpd][4];
#pragma unroll
    for (int q = 0; q < kUpd; ++q) {
      const int t = mb + 1 + wave + kWaves * q;
      const int tc = t < nt ? t : nt - 1;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        ub[q][kk] = U[(int64_t)(gcol + 4 * kk + (lane >> 4)) * a.ldu + a.i1 + 16 * tc + (lane & 15)];
    }
    {
      const double* ud = Ud + buf * 256;
      double w[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) w[j] = S[r * sp + c0 + j];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        // the group's triangle of U and its reciprocal pivots
        double T[D][D], inv[D];
#pragma unroll
        for (int i = 0; i < D; ++i) {
          inv[i] = Id[buf * 16 + g * D + i];
#pragma unroll
          for (int k = i + 1; k < D; ++k) T[i][k] = ud[(g * D + i) * 16 + g * D + k];
        }
        // losses of this lane's entries, ascending index: a later entry wins only if strictly smaller
        double best = __builtin_inf();
        int bidx = 0x7fffffff;
#pragma unroll
        for (int s = 0; s < kSlots; ++s) {
          const int k = l32 + 32 * s;
          double rem[D], loss = 0.0;
#pragma unroll
          for (int i = 0; i < D; ++i) rem[i] = w[g * D + i] - cb[s][i];
#pragma unroll
          for (int i = 0; i < D; ++i) {
            const double e = rem[i] * inv[i];
#pragma unroll
            for (int kx = i + 1; kx < D; ++kx) rem[kx] = fma(-e, T[i][kx], rem[kx]);
            loss = fma(e, e, loss);
          }
          const bool take = k < a.K && loss < best;
          best = take ? loss : best;
          bidx = take ? k : bidx;
        }
        take_smaller<1>(best, bidx);
        take_smaller<2>(best, bidx);
        take_smaller<4>(best, bidx);
        take_smaller<8>(best, bidx);
        take_smaller<16>(best, bidx);
        // every lane of the half-wave now holds the assigned index; its entry comes from the lane that owns it
        double q[D], e[D];
        {
          const int owner = ((lane & 32) | (bidx & 31)) << 2, slot = bidx >> 5;
#pragma unroll
          for (int i = 0; i < D; ++i) {
            double mine = cb[0][i];
#pragma unroll
            for (int s = 1; s < kSlots; ++s) mine = (slot == s) ? cb[s][i] : mine;
            const int lo = __builtin_amdgcn_ds_bpermute(owner, __double2loint(mine));
            const int hi = __builtin_amdgcn_ds_bpermute(owner, __double2hiint(mine));
            q[i] = __hiloint2double(hi, lo);
          }
        }
        {
          double rem[D];
#pragma unroll
          for (int i = 0; i < D; ++i) rem[i] = w[g * D + i] - q[i];
#pragma unroll
          for (int i = 0; i < D; ++i) {
            e[i] = rem[i] * inv[i];
#pragma unroll
            for (int kx = i + 1; kx < D; ++kx) rem[kx] = fma(-e[i], T[i][kx], rem[kx]);
          }
        }
        // the group's errors onto the later columns of the mini-block
#pragma unroll
        for (int c = (g + 1) * D; c < 16; ++c) {
#pragma unroll
          for (int i = 0; i < D; ++i) w[c] = fma(-e[i], ud[(g * D + i) * 16 + c], w[c]);
        }
        if (l32 == 0) {
#pragma unroll
          for (int i = 0; i < D; ++i) {
            Em[(g * D + i) * kRows + r] = e[i];
            Qm[(g * D + i) * 17 + r] = q[i];
            err2 = fma(e[i], e[i], err2);
          }
          It[r * gpb + mb * G + g] = (uint8_t)bidx;
        }
      }
    }
    __syncthreads();
    // push the 16 new errors onto the later tiles of the block
#pragma unroll
    for (int q = 0; q < kUpd; ++q) {
      const int t = mb + 1 + wave + kWaves * q;
      if (t < nt) {
        f64x4 d = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const double av = Em[(4 * kk + (lane >> 4)) * kRows + (lane & 15)];
          d = __builtin_amdgcn_mfma_f64_16x16x4f64(av, ub[q][kk], d, 0, 0, 0);
        }
        double sv[4];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) sv[rr] = S[(4 * rr + (lane >> 4)) * sp + 16 * t + (lane & 15)];
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) S[(4 * rr + (lane >> 4)) * sp + 16 * t + (lane & 15)] = sv[rr] - d[rr];
      }
    }
    if (tid >= 256) {
      const int e = tid - 256;
      a.errT[(int64_t)(gcol + (e >> 4)) * a.mpad + row0 + (e & 15)] = Em[e];
      const int rr = e >> 4, j = e & 15;
      if (a.Wq && row0 + rr < a.m) a.Wq[(int64_t)(row0 + rr) * a.n + gcol + j] = Qm[j * 17 + rr];
    }
    if (mb + 1 < nt) {
      if (tid < 256) Ud[(buf ^ 1) * 256 + tid] = ud_next;
      if (tid < 16) Id[(buf ^ 1) * 16 + tid] = id_next;
    }
    __syncthreads();
  }

  // ---- outputs of the block
  const int ng = a.n / D;
  for (int e = tid; e < kRows * gpb; e += kThreads) {
    const int rr = e / gpb, c = e - rr * gpb;
    if (row0 + rr < a.m) a.indices[(int64_t)(row0 + rr) * ng + a.i1 / D + c] = It[rr * gpb + c];
  }
  if (a.row_err2 && (lane & 31) == 0 && row0 + r < a.m) {
    if (a.i1 == 0)
      a.row_err2[row0 + r] = err2;
    else
      a.row_err2[row0 + r] += err2;
  }
}

size_t vq_lds_bytes(int bw) {
  return (size_t)(4 * kRows * bw + 256 + 272 + 512 + 32) * sizeof(double) + (size_t)kRows * bw;
}

template <int DT, int NT, int D>
ptq_status vq_launch_block(const VqArgs& a, hipStream_t st) {
  if (!lds_opt_in<vq_block_kernel<DT, NT, D>>((int)vq_lds_bytes(16 * NT))) return PTQ_ERR_HIP;
  vq_block_kernel<DT, NT, D><<<(unsigned)ceil_div(a.m, kRows), kThreads, vq_lds_bytes(a.bw), st>>>(a);
  return PTQ_OK;
}

template <int DT, int D>
ptq_status vq_run_blocks(VqArgs a, int block, hipStream_t st) {
  for (int i1 = 0; i1 < a.n; i1 += block) {
    a.i1 = i1;
    a.bw = (a.n - i1 < block) ? a.n - i1 : block;
    const ptq_status rc = (a.bw <= 128) ? vq_launch_block<DT, 8, D>(a, st) : vq_launch_block<DT, 16, D>(a, st);
    if (rc != PTQ_OK) return rc;
  }
  return PTQ_OK;
}

template <int DT>
ptq_status vq_run_dim(const VqArgs& a, int d, int block, hipStream_t st) {
  switch (d) {
    case 1: return vq_run_blocks<DT, 1>(a, block, st);
    case 2: return vq_run_blocks<DT, 2>(a, block, st);
    case 4: return vq_run_blocks<DT, 4>(a, block, st);
    default: return PTQ_ERR_ARG;
  }
}

}  // namespace

ptq_status quantize_vq_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* U,
                              int64_t ldu, const uint8_t* dead_mask, const float* codebook, int entries, int dim,
                              int block, uint8_t* indices, double* Wq, double* row_err2, void* ws, size_t ws_bytes,
                              hipStream_t st) {
  if (m == 0 || n == 0) return PTQ_OK;
  if (ws_bytes < quantize_workspace_bytes(m, n)) return PTQ_ERR_WORKSPACE;
  VqArgs a;
  a.W = W;
  a.ldw = ldw;
  a.m = (int)m;
  a.n = (int)n;
  a.mpad = (int)(ceil_div(m, kRowAlign) * kRowAlign);
  a.U = U;
  a.ldu = ldu;
  a.dead = dead_mask;
  a.errT = static_cast<double*>(ws);
  a.invd = reinterpret_cast<double*>(static_cast<char*>(ws) + align_up((size_t)n * (size_t)a.mpad * sizeof(double), 256));
  a.codebook = codebook;
  a.K = entries;
  a.i1 = 0;
  a.bw = 0;
  a.indices = indices;
  a.Wq = Wq;
  a.row_err2 = row_err2;
  vq_inv_diag_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(U, ldu, (int)n, const_cast<double*>(a.invd));
  PTQ_HIP_CHECK_LAUNCH();
  ptq_status rc;
  switch (wdt) {
    case PTQ_F32: rc = vq_run_dim<PTQ_F32>(a, dim, block, st); break;
    case PTQ_BF16: rc = vq_run_dim<PTQ_BF16>(a, dim, block, st); break;
    case PTQ_F64: rc = vq_run_dim<PTQ_F64>(a, dim, block, st); break;
    default: return PTQ_ERR_DTYPE;
  }
  if (rc != PTQ_OK) return rc;
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
