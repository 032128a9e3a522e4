// LoPRo's pre-conditioning of the layer solve (paper Sec. 3.2): column order (Eq. 5), the
// partial block Walsh-Hadamard rotation of a weight-shaped matrix, R' = R P Q (Eq. 6), its
// way back, Rq Q^T P^T (Eq. 7), and the rotated Hessian H' = Q^T P^T H P Q (Eq. 8).
//
// All of it is memory-bound: every element is read and written once or twice and takes
// log2(b_H) additions on the way.  A row transform stages the row in LDS (so that the
// column gather / scatter never touches HBM at element granularity), and a wave transforms
// 256 consecutive columns at a time, four per lane: two butterfly stages in registers, up to
// six across lanes.  The column direction of H' works on tiles of b_H rows x 32 columns in
// LDS with two register passes of at most sixteen points each.
#include "common.h"

namespace ptq {
namespace {

__device__ __forceinline__ double lane_xor(double v, int mask) {
  const int lo = __shfl_xor(__double2loint(v), mask);
  const int hi = __shfl_xor(__double2hiint(v), mask);
  return __hiloint2double(hi, lo);
}

// Walsh-Hadamard transform (natural order, unscaled) of blocks of `bh` consecutive elements of a
// 256-element chunk held four per lane, element 4 * lane + i in v[i]; bh = 2^lg, 4 <= bh <= 256.
__device__ __forceinline__ void fwht_chunk(double (&v)[4], int lg, int lane) {
  {
    const double a = v[0] + v[1], b = v[0] - v[1], c = v[2] + v[3], d = v[2] - v[3];
    v[0] = a + c;
    v[1] = b + d;
    v[2] = a - c;
    v[3] = b - d;
  }
  for (int s = 0; s + 2 < lg; ++s) {
    const bool upper = (lane >> s) & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double p = lane_xor(v[i], 1 << s);
      v[i] = upper ? p - v[i] : v[i] + p;
    }
  }
}

__device__ __forceinline__ int ilog2(int x) { return 31 - __clz(x); }

// ---- column order ------------------------------------------------------------------------
constexpr int kOrderSplits = 64;   // row slices whose partial sums are added in a fixed order

template <int DT>
__global__ __launch_bounds__(256) void abs_colsum_kernel(const void* __restrict__ R, int64_t ldr, int m,
                                                         int n, double* __restrict__ partial) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= n) return;
  double s = 0.0;
  for (int r = blockIdx.y; r < m; r += kOrderSplits) s += fabs(load_as_f64<DT>(R, (int64_t)r * ldr + c));
  partial[(int64_t)blockIdx.y * n + c] = s;
}

__global__ __launch_bounds__(256) void keys_kernel(const double* __restrict__ partial, const double* __restrict__ H,
                                                   int64_t ldh, int m, int n, double* __restrict__ keys) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= n) return;
  double s = 0.0;
  for (int k = 0; k < kOrderSplits; ++k) s += partial[(int64_t)k * n + c];
  const double a = s / (double)m, d = H[(int64_t)c * ldh + c];
  keys[c] = (a != 0.0) ? d / a : (d > 0.0 ? __builtin_inf() : 0.0);
}

// perm[rank] = column, rank = number of columns that come before it (ties: lower index first).
// A workgroup ranks 16 columns; the comparisons against all n keys are split over sixteen lanes
// per column and the sixteen counts are added with shuffles.  The keys are staged in LDS in
// pieces of kRankStage (every lane reads all of them; from global memory the loop is a chain of
// load latencies).
constexpr int kRankStage = 4096;
__global__ __launch_bounds__(256) void rank_kernel(const double* __restrict__ keys, int n, int descending,
                                                   int32_t* __restrict__ perm) {
  __shared__ double ks[kRankStage];
  const int i = blockIdx.x * 16 + (threadIdx.x >> 4), sl = threadIdx.x & 15;
  const double ki = i < n ? keys[i] : 0.0;
  int rank = 0;
  for (int j0 = 0; j0 < n; j0 += kRankStage) {
    const int cnt = min(kRankStage, n - j0);
    __syncthreads();
    for (int j = threadIdx.x; j < cnt; j += 256) ks[j] = keys[j0 + j];
    __syncthreads();
#pragma unroll 8
    for (int j = sl; j < cnt; j += 16) {
      const double kj = ks[j];
      const bool first = descending ? (kj > ki) : (kj < ki);
      rank += (first || (kj == ki && j0 + j < i)) ? 1 : 0;
    }
  }
  rank += __shfl_xor(rank, 1);
  rank += __shfl_xor(rank, 2);
  rank += __shfl_xor(rank, 4);
  rank += __shfl_xor(rank, 8);
  if (i < n && sl == 0) perm[rank] = i;
}

// ---- row transforms ----------------------------------------------------------------------
// MODE 0:  out[row, c] = sum_c' in[src_row, perm[c']] Q[c', c]     (gather, then rotate)
// MODE 1:  out[row, perm[c]] = sum_c' in[row, c'] Q[c, c']          (rotate, then scatter)
// One workgroup per row; the row is staged in LDS in its storage type (MODE 0) resp. as float64
// (MODE 1).  row_perm (MODE 0 only, may be null) picks the source row.
// (256 threads, or 1024 when the staged row is so large that only one workgroup fits a CU.)
// OT: float64, or (MODE 0 only) float32 for activations on their way into the stored layer.
template <int DT, int MODE, typename OT>
__global__ __launch_bounds__(1024) void row_rotate_kernel(const void* __restrict__ in, int64_t ldi, int n,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ row_perm, int b_I, int b_H,
                                                         OT* __restrict__ out, int64_t ldo) {
  static_assert(MODE == 0 || sizeof(OT) == sizeof(double), "the scatter form writes float64");
  extern __shared__ __attribute__((aligned(16))) char rowbuf[];
  using ST = typename StoredType<DT>::type;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nthr = blockDim.x, nwave = nthr >> 6;
  const int row = blockIdx.x;
  const int lg = ilog2(b_H);
  const double scale = 1.0 / sqrt((double)b_H);
  const int nchunk_id = (b_I + 255) / 256;                 // chunks of the identity part
  const int nchunk = nchunk_id + (n - b_I + 255) / 256;    // ... plus those of the rotated part
  if (MODE == 0) {
    const int64_t src = row_perm ? row_perm[row] : row;
    ST* buf = reinterpret_cast<ST*>(rowbuf);
    for (int c = tid; c < n; c += nthr) buf[c] = load_stored<DT>(in, src * ldi + c);
    __syncthreads();
    for (int k = wave; k < nchunk; k += nwave) {
      const bool ident = k < nchunk_id;
      const int cs = ident ? 256 * k : b_I + 256 * (k - nchunk_id);
      const int ce = ident ? b_I : n;
      const int c = cs + 4 * lane;
      double v[4] = {0.0, 0.0, 0.0, 0.0};
      if (c < ce) {
        const int4 p = *reinterpret_cast<const int4*>(perm + c);
        v[0] = stored_to_f64<DT>(buf[p.x]);
        v[1] = stored_to_f64<DT>(buf[p.y]);
        v[2] = stored_to_f64<DT>(buf[p.z]);
        v[3] = stored_to_f64<DT>(buf[p.w]);
      }
      if (!ident) {
        fwht_chunk(v, lg, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] *= scale;
      }
      if (c < ce) {
        OT* o = out + (int64_t)row * ldo + c;
        if constexpr (sizeof(OT) == sizeof(double)) {
          *reinterpret_cast<double2*>(o) = double2{v[0], v[1]};
          *reinterpret_cast<double2*>(o + 2) = double2{v[2], v[3]};
        } else {
          *reinterpret_cast<float4*>(o) = make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
        }
      }
    }
  } else {
    double* buf = reinterpret_cast<double*>(rowbuf);
    const double* irow = static_cast<const double*>(in) + (int64_t)row * ldi;
    for (int k = wave; k < nchunk; k += nwave) {
      const bool ident = k < nchunk_id;
      const int cs = ident ? 256 * k : b_I + 256 * (k - nchunk_id);
      const int ce = ident ? b_I : n;
      const int c = cs + 4 * lane;
      double v[4] = {0.0, 0.0, 0.0, 0.0};
      if (c < ce) {
        const double2 a = *reinterpret_cast<const double2*>(irow + c);
        const double2 b = *reinterpret_cast<const double2*>(irow + c + 2);
        v[0] = a.x;
        v[1] = a.y;
        v[2] = b.x;
        v[3] = b.y;
      }
      if (!ident) {
        fwht_chunk(v, lg, lane);
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] *= scale;
      }
      if (c < ce) {
        const int4 p = *reinterpret_cast<const int4*>(perm + c);
        buf[p.x] = v[0];
        buf[p.y] = v[1];
        buf[p.z] = v[2];
        buf[p.w] = v[3];
      }
    }
    __syncthreads();
    for (int c = tid; c < n; c += nthr) out[(int64_t)row * ldo + c] = (OT)buf[c];
  }
}

// ---- Hessian -----------------------------------------------------------------------------
// Full symmetric copy of a matrix given by its upper triangle, 32 x 32 tiles through LDS.
__global__ __launch_bounds__(256) void symmetrize_kernel(const double* __restrict__ H, int64_t ldh, int n,
                                                         double* __restrict__ Hs) {
  __shared__ double t[32][33];
  const int I = blockIdx.y, J = blockIdx.x;
  if (I > J) return;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < 32; r += 8) {
    const int i = I * 32 + r, j = J * 32 + tx;
    double v = 0.0;
    if (i < n && j < n) v = (i <= j) ? H[(int64_t)i * ldh + j] : H[(int64_t)j * ldh + i];
    t[r][tx] = v;
    if (i < n && j < n) Hs[(int64_t)i * n + j] = v;
  }
  __syncthreads();
  if (I == J) return;
  for (int r = ty; r < 32; r += 8) {
    const int i = J * 32 + r, j = I * 32 + tx;
    if (i < n && j < n) Hs[(int64_t)i * n + j] = t[tx][r];
  }
}

// In-place Walsh-Hadamard transform (scaled) down the columns, in blocks of b_H rows starting at
// row b_I: a workgroup takes b_H rows x 32 columns.  With r = 16 a + b inside a block, the first
// pass transforms over b (16 consecutive rows), the second over a (rows 16 apart).
__device__ __forceinline__ void fwht16(double (&x)[16], int lg) {
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    if (s < lg) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        if (!(i & (1 << s))) {
          const double a = x[i], b = x[i | (1 << s)];
          x[i] = a + b;
          x[i | (1 << s)] = a - b;
        }
      }
    }
  }
}

__global__ __launch_bounds__(512) void col_rotate_kernel(double* __restrict__ A, int64_t lda, int n, int b_I,
                                                         int b_H) {
  extern __shared__ double tile[];   // [b_H][33]
  const int tid = threadIdx.x;
  const int r0 = b_I + blockIdx.y * b_H, c0 = blockIdx.x * 32;
  const int lg = ilog2(b_H);
  const double scale = 1.0 / sqrt((double)b_H);
  const int cx = tid & 31;
  for (int r = tid >> 5; r < b_H; r += 16)
    tile[r * 33 + cx] = (c0 + cx < n) ? A[(int64_t)(r0 + r) * lda + c0 + cx] : 0.0;
  __syncthreads();
  const int groups = b_H / 16;   // 1 .. 16
  // pass 1: over b (bits 0..3 of the row index), groups x 32 column vectors
  for (int g = tid >> 5; g < groups; g += 16) {
    double x[16];
#pragma unroll
    for (int b = 0; b < 16; ++b) x[b] = tile[(16 * g + b) * 33 + cx];
    fwht16(x, 4);
#pragma unroll
    for (int b = 0; b < 16; ++b) tile[(16 * g + b) * 33 + cx] = x[b];
  }
  __syncthreads();
  // pass 2: over a (bits 4.. of the row index), 16 x 32 column vectors of `groups` points
  for (int b = tid >> 5; b < 16; b += 16) {
    double x[16];
#pragma unroll
    for (int a = 0; a < 16; ++a) x[a] = a < groups ? tile[(16 * a + b) * 33 + cx] : 0.0;
    fwht16(x, lg - 4);
#pragma unroll
    for (int a = 0; a < 16; ++a)
      if (a < groups) tile[(16 * a + b) * 33 + cx] = x[a] * scale;
  }
  __syncthreads();
  for (int r = tid >> 5; r < b_H; r += 16)
    if (c0 + cx < n) A[(int64_t)(r0 + r) * lda + c0 + cx] = tile[r * 33 + cx];
}

size_t stored_size(ptq_dtype dt) { return dt == PTQ_BF16 ? 2 : (dt == PTQ_F32 ? 4 : 8); }

template <int MODE, typename OT>
ptq_status launch_row_rotate(const void* in, ptq_dtype dt, int64_t ldi, int64_t rows, int64_t n,
                             const int32_t* perm, const int32_t* row_perm, int b_I, int b_H, OT* out,
                             int64_t ldo, hipStream_t st) {
  const size_t lds = (size_t)n * (MODE == 0 ? stored_size(dt) : sizeof(double));
  if (lds > 160 * 1024) return PTQ_ERR_SHAPE;
#define PTQ_ROW_CASE(DT)                                                                                   \
  {                                                                                                        \
    if (!lds_opt_in<row_rotate_kernel<DT, MODE, OT>>(160 * 1024)) return PTQ_ERR_HIP;                          \
    row_rotate_kernel<DT, MODE, OT><<<(unsigned)rows, lds > 40 * 1024 ? 1024 : 256, lds, st>>>(                \
        in, ldi, (int)n, perm, row_perm, b_I, b_H, out, ldo);                                              \
  }
  switch (dt) {
    case PTQ_F32: PTQ_ROW_CASE(PTQ_F32) break;
    case PTQ_BF16: PTQ_ROW_CASE(PTQ_BF16) break;
    case PTQ_F64: PTQ_ROW_CASE(PTQ_F64) break;
    default: return PTQ_ERR_DTYPE;
  }
#undef PTQ_ROW_CASE
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace

size_t lopro_order_workspace_bytes(int64_t n) {
  return align_up((size_t)(kOrderSplits + 1) * (size_t)n * sizeof(double), 256);
}

size_t lopro_hessian_workspace_bytes(int64_t n) {
  return align_up((size_t)n * (size_t)n * sizeof(double), 256);
}

ptq_status lopro_order_launch(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n, const double* H,
                              int64_t ldh, int descending, int32_t* perm, double* keys, void* ws,
                              hipStream_t st) {
  double* partial = static_cast<double*>(ws);
  double* k = keys ? keys : partial + (size_t)kOrderSplits * n;
  dim3 g((unsigned)ceil_div(n, 256), kOrderSplits);
  switch (rdt) {
    case PTQ_F32: abs_colsum_kernel<PTQ_F32><<<g, 256, 0, st>>>(R, ldr, (int)m, (int)n, partial); break;
    case PTQ_BF16: abs_colsum_kernel<PTQ_BF16><<<g, 256, 0, st>>>(R, ldr, (int)m, (int)n, partial); break;
    case PTQ_F64: abs_colsum_kernel<PTQ_F64><<<g, 256, 0, st>>>(R, ldr, (int)m, (int)n, partial); break;
    default: return PTQ_ERR_DTYPE;
  }
  keys_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(partial, H, ldh, (int)m, (int)n, k);
  rank_kernel<<<(unsigned)ceil_div(n, 16), 256, 0, st>>>(k, (int)n, descending, perm);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status lopro_rotate_weight_launch(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                      const int32_t* perm, int b_I, int b_H, double* Rout, int64_t ldo,
                                      hipStream_t st) {
  return launch_row_rotate<0, double>(R, rdt, ldr, m, n, perm, nullptr, b_I, b_H, Rout, ldo, st);
}

ptq_status lopro_rotate_input_launch(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t n,
                                     const int32_t* perm, int b_I, int b_H, float* Xout, int64_t ldo,
                                     hipStream_t st) {
  return launch_row_rotate<0, float>(X, xdt, ldx, tokens, n, perm, nullptr, b_I, b_H, Xout, ldo, st);
}

ptq_status lopro_unrotate_weight_launch(const double* Rq, int64_t ldq, int64_t m, int64_t n,
                                        const int32_t* perm, int b_I, int b_H, double* Wout, int64_t ldo,
                                        hipStream_t st) {
  return launch_row_rotate<1, double>(Rq, PTQ_F64, ldq, m, n, perm, nullptr, b_I, b_H, Wout, ldo, st);
}

ptq_status lopro_rotate_hessian_launch(const double* H, int64_t ldh, int64_t n, const int32_t* perm, int b_I,
                                       int b_H, double* Hout, int64_t ldo, void* ws, hipStream_t st) {
  double* Hs = static_cast<double*>(ws);
  dim3 gs((unsigned)ceil_div(n, 32), (unsigned)ceil_div(n, 32));
  symmetrize_kernel<<<gs, 256, 0, st>>>(H, ldh, (int)n, Hs);
  // rows: Hout[r, :] = (row perm[r] of H, columns gathered by perm) rotated
  ptq_status rc = launch_row_rotate<0, double>(Hs, PTQ_F64, n, n, n, perm, perm, b_I, b_H, Hout, ldo, st);
  if (rc != PTQ_OK) return rc;
  // columns: H' = Q^T (that)
  if (n > b_I) {
    if (!lds_opt_in<col_rotate_kernel>(256 * 33 * 8)) return PTQ_ERR_HIP;
    dim3 gc((unsigned)ceil_div(n, 32), (unsigned)((n - b_I) / b_H));
    col_rotate_kernel<<<gc, 512, (size_t)b_H * 33 * sizeof(double), st>>>(Hout, ldo, (int)n, b_I, b_H);
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
