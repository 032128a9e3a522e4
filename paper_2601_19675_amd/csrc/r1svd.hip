// Scaled rank-one randomized sketching (paper Sec. 3.3, Eq. 9-11; Algorithm 1, inner loop)
// and the activation scale that precedes it.
//
// One rank costs  y = (A A^T)^it A v,  p = A^T y.  Written as  y = A (A^T A)^it v  this is
// it + 1 applications of "u = A v, z = A^T u" to the same matrix, and both products of one
// application can be taken from ONE pass over A.  So a rank reads A  it + 1  times instead of
// 2 it + 2  times, and every sum has a fixed order (results are reproducible).
//
// The loop exists in five forms, chosen by shape and type (r1svd_launch); resident and stream are
// in r1svd_bf16.hip, the helpers all forms share in r1svd_device.h:
//   tile      A (float32) in the registers of 256 workgroups, a 256 x 256 tile each, for the whole
//             loop; partial sums travel as tagged words, no barrier inside an application
//   resident  a bfloat16 W too large for that: W itself stays on the chip (registers + LDS) in
//             P x Q tiles and A = W diag(s) - stored rank-one terms is never formed; tagged words
//   stream    a bfloat16 W too large for the chip: the same implicit products, row blocks of W
//             streamed from memory in every application, grid barriers
//   rows      any other type: row blocks of the float32 A, deflated in place, streamed; one launch
//   steps     the same row blocks as one launch per application and per partial sum, when the
//             device cannot hold a cooperative launch
// In the row-block forms a workgroup owns R complete rows, keeps them in registers, finishes its
// R entries of u = A v (a reduction inside the workgroup) and multiplies the same registers by
// those entries to get its share of z = A^T u, which it writes as a partial vector.
//
// Arithmetic: the matrix and the vector v of an application are float32 (bfloat16 weights are
// exact in it), and so are the products and the short sums a thread forms from its own columns
// (for u) or rows (for z); everything that is added across threads, workgroups or row blocks is
// float64, as are the norms and the values that get rounded to e4m3 / fp16.  That keeps the noise
// at the level the float32 storage of A sets anyway.  Vectors grow by sigma_1^2 per application;
// v is z times a power of two (exact) taken from the size of z, so the printed formula is
// evaluated as it stands.
#include "r1svd_device.h"

#include <cstdlib>
#include <cstring>

namespace ptq {
namespace {

using namespace r1svd_detail;

// ---- activation magnitude and scale (Algorithm 1) ------------------------------------------
constexpr int kAbsSlices = 256;    // token slices whose partial sums are added in a fixed order
constexpr int kAbsCols = 512;      // columns per workgroup: 64 threads x 8, times 4 token lanes

template <int DT>
__global__ __launch_bounds__(256) void abs_sum_kernel(const void* __restrict__ X, int64_t ldx, int64_t t, int n,
                                                      double* __restrict__ partial) {
  const int cl = threadIdx.x & 63, tl = threadIdx.x >> 6;
  const int c0 = blockIdx.x * kAbsCols + cl * 8;
  const int64_t per = (t + kAbsSlices - 1) / kAbsSlices;
  const int64_t k0 = (int64_t)blockIdx.y * per, k1 = (k0 + per < t) ? k0 + per : t;
  double acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.0;
  if (c0 < n) {   // n is a multiple of 8
    for (int64_t k = k0 + tl; k < k1; k += 4) {
      if constexpr (DT == PTQ_BF16) {
        const uint4 q = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(X) + k * ldx + c0);
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          acc[2 * c] += (double)fabsf(__uint_as_float(w[c] << 16));
          acc[2 * c + 1] += (double)fabsf(__uint_as_float(w[c] & 0xffff0000u));
        }
      } else {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(X) + k * ldx + c0);
        const float4 a = p[0], b = p[1];
        acc[0] += (double)fabsf(a.x); acc[1] += (double)fabsf(a.y);
        acc[2] += (double)fabsf(a.z); acc[3] += (double)fabsf(a.w);
        acc[4] += (double)fabsf(b.x); acc[5] += (double)fabsf(b.y);
        acc[6] += (double)fabsf(b.z); acc[7] += (double)fabsf(b.w);
      }
    }
  }
  __shared__ double red[4][kAbsCols];
#pragma unroll
  for (int c = 0; c < 8; ++c) red[tl][cl * 8 + c] = acc[c];
  __syncthreads();
  for (int c = threadIdx.x; c < kAbsCols; c += 256) {
    const int col = blockIdx.x * kAbsCols + c;
    if (col < n) partial[(int64_t)blockIdx.y * n + col] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
  }
}

__global__ __launch_bounds__(256) void abs_sum_finish_kernel(const double* __restrict__ partial, int n,
                                                             double* __restrict__ asum) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= n) return;
  double s = 0.0;
  for (int k = 0; k < kAbsSlices; ++k) s += partial[(int64_t)k * n + c];
  asum[c] += s;
}

// s_j = Xbar_j^2.5 / sqrt(max Xbar * min Xbar) over the channels with Xbar > 0; 1 elsewhere.
__global__ __launch_bounds__(1024) void scale_kernel(const double* __restrict__ asum, double tokens, int n,
                                                     double* __restrict__ s) {
  __shared__ double shi[16], slo[16];
  double hi = 0.0, lo = __builtin_inf();
  for (int c = threadIdx.x; c < n; c += 1024) {
    const double x = asum[c] / tokens;
    if (x > 0.0) { hi = fmax(hi, x); lo = fmin(lo, x); }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    hi = fmax(hi, __shfl_xor(hi, o));
    lo = fmin(lo, __shfl_xor(lo, o));
  }
  if ((threadIdx.x & 63) == 0) { shi[threadIdx.x >> 6] = hi; slo[threadIdx.x >> 6] = lo; }
  __syncthreads();
  hi = shi[0]; lo = slo[0];
  for (int w = 1; w < 16; ++w) { hi = fmax(hi, shi[w]); lo = fmin(lo, slo[w]); }
  const double den = sqrt(hi * lo);
  for (int c = threadIdx.x; c < n; c += 1024) {
    const double x = asum[c] / tokens;
    s[c] = x > 0.0 ? x * x * sqrt(x) / den : 1.0;
  }
}

__global__ void clear_counter_kernel(unsigned* counter) {
  if (threadIdx.x == 0) *counter = 0u;
}

// ---- W_s = W diag(s) ---------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(256) void scale_weight_kernel(const void* __restrict__ W, int64_t ldw, int m, int n,
                                                           const double* __restrict__ s, float* __restrict__ A) {
  const int nb = (n + 1023) / 1024;
  const int c = ((int)(blockIdx.x % nb) * 256 + threadIdx.x) * 4;
  const int row = blockIdx.x / nb;
  if (c >= n) return;
  float4 o;
  o.x = (float)(load_as_f64<DT>(W, (int64_t)row * ldw + c) * s[c]);
  o.y = (float)(load_as_f64<DT>(W, (int64_t)row * ldw + c + 1) * s[c + 1]);
  o.z = (float)(load_as_f64<DT>(W, (int64_t)row * ldw + c + 2) * s[c + 2]);
  o.w = (float)(load_as_f64<DT>(W, (int64_t)row * ldw + c + 3) * s[c + 3]);
  *reinterpret_cast<float4*>(A + (int64_t)row * n + c) = o;
}

// ---- one application  u = A v,  z = A^T u -----------------------------------------------------
struct PassArgs {
  float* A;                 // m x n, leading dimension n
  int m, n;
  const float* vin;         // the sketch vector (first application of a rank) or the previous z
  const double* rescale;    // power of two applied to vin (null: 1)
  double* u;                // m
  double* unrm2;            // per workgroup: sum of squares of its entries of u
  float* zpart;             // one partial z per workgroup, see store_partial for the layout
  // deflation by the previous rank's stored triplet, applied to A while it is loaded
  const double* sigma;      // null: none
  const double* ud;         // m
  const double* vd;         // n
};

// A block of R rows of A in the registers of a workgroup of T threads: a thread owns 4 adjacent
// columns in each of NS sweeps of 4 T columns.
// COH: the vectors come from other workgroups of the same launch (see load_dev).
template <int T, int NS, int R, bool COH = false>
struct RowBlock {
  float w[NS][R][4];

  static __device__ __forceinline__ double vec(const double* p) { return COH ? load_dev(p) : *p; }

  // Loads rows row0 .. row0+R-1 (zeros outside the matrix).  With `deflate` the previous rank's
  // stored triplet (sg, ud, vd) is subtracted on the way (float64 arithmetic, one rounding to
  // float32) and the result is stored back.
  __device__ __forceinline__ void load(float* A, int m, int n, int row0, bool deflate, double sg, const double* ud,
                                       const double* vd) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 4 * (tid + T * s);
      double dv[4] = {0.0, 0.0, 0.0, 0.0};
      if (deflate && col < n) {
#pragma unroll
        for (int c = 0; c < 4; ++c) dv[c] = sg * vec(vd + col + c);
      }
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const int row = row0 + i;
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col < n && row < m) {
          float4* p = reinterpret_cast<float4*>(A + (int64_t)row * n + col);
          q = *p;
          if (deflate) {
            const double ui = vec(ud + row);
            q.x = (float)((double)q.x - ui * dv[0]);
            q.y = (float)((double)q.y - ui * dv[1]);
            q.z = (float)((double)q.z - ui * dv[2]);
            q.w = (float)((double)q.w - ui * dv[3]);
            *p = q;
          }
        }
        w[s][i][0] = q.x; w[s][i][1] = q.y; w[s][i][2] = q.z; w[s][i][3] = q.w;
      }
    }
  }

  // u = (block) v for the R rows, left in ush[0..R) (and in u_out, if not null); then
  // zacc += (block)^T u.  v is vin times the power of two rs.
  // Returns the sum of squares of the R entries of u (valid in thread 0).
  // red: T/64 x R doubles, ush: R doubles, stage: T/64 x 512 floats of LDS.  Contains two workgroup barriers.
  __device__ __forceinline__ double apply(const float* vin, float rs, int m, int n, int row0, double* u_out,
                                          double (&zacc)[NS][4], double* red, double* ush, float* stage) {
    constexpr int kWaves = T / kWave;
    const int tid = threadIdx.x;
    float us[R];
#pragma unroll
    for (int i = 0; i < R; ++i) us[i] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 4 * (tid + T * s);
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (col < n) v = *reinterpret_cast<const float4*>(vin + col);
      v.x *= rs; v.y *= rs; v.z *= rs; v.w *= rs;
#pragma unroll
      for (int i = 0; i < R; ++i)
        us[i] = fmaf(w[s][i][3], v.w, fmaf(w[s][i][2], v.z, fmaf(w[s][i][1], v.y, fmaf(w[s][i][0], v.x, us[i]))));
    }
    wave_row_sums_into<R>(us, red, stage + (tid >> 6) * 512);
    __syncthreads();
    if (tid < R) {
      double t = 0.0;
#pragma unroll
      for (int wv = 0; wv < kWaves; ++wv) t += red[wv * R + tid];
      ush[tid] = t;
      if (u_out && row0 + tid < m) u_out[row0 + tid] = t;
    }
    __syncthreads();
    double nrm2 = 0.0;
    if (tid == 0) {
#pragma unroll
      for (int i = 0; i < R; ++i) nrm2 = fma(ush[i], ush[i], nrm2);
    }
    float uf[R];
#pragma unroll
    for (int i = 0; i < R; ++i) uf[i] = (float)ush[i];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      float zt[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) zt[c] = fmaf(w[s][i][c], uf[i], zt[c]);
#pragma unroll
      for (int c = 0; c < 4; ++c) zacc[s][c] += (double)zt[c];
    }
    return nrm2;
  }
};

// Partial vectors are stored as float32 in blocks of kReduceCols columns, [column block][workgroup]
// [column], so that the sum over workgroups reads contiguous memory.
template <int T, int NS, bool COH = false>
__device__ __forceinline__ void store_partial(const double (&zacc)[NS][4], float* zpart, int n, int part,
                                              int parts) {
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int col = 4 * ((int)threadIdx.x + T * s);
    if (col < n) {
      float* o = zpart + ((int64_t)(col / kReduceCols) * parts + part) * kReduceCols + col % kReduceCols;
      const float x = (float)zacc[s][0], y = (float)zacc[s][1], z = (float)zacc[s][2], w = (float)zacc[s][3];
      if (COH) store_dev4(o, x, y, z, w);
      else *reinterpret_cast<float4*>(o) = make_float4(x, y, z, w);
    }
  }
}

template <int T, int NS, int R, bool DEFLATE>
__global__ __launch_bounds__(T) void pass_kernel(PassArgs a) {
  __shared__ double red[T / kWave * R];
  __shared__ double ush[R];
  __shared__ float stage[T / kWave * 512];
  double zacc[NS][4];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int c = 0; c < 4; ++c) zacc[s][c] = 0.0;
  double unrm2 = 0.0;   // thread 0 only
  const float rs = a.rescale ? (float)*a.rescale : 1.f;
  const int tiles = (a.m + R - 1) / R;

  // a workgroup walks over row blocks and keeps adding to the same partial z, so that the
  // number of partial vectors is the number of workgroups, whatever the number of rows
  for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    // the vectors are re-read (from cache) for every row block: kept in registers across the
    // loop they would take 8 per sweep and push the block's own data out
    const float* vin = a.vin;
    const double* vd = a.vd;
    asm volatile("" : "+s"(vin), "+s"(vd));
    RowBlock<T, NS, R> blk;
    blk.load(a.A, a.m, a.n, tile * R, DEFLATE, DEFLATE ? *a.sigma : 0.0, a.ud, vd);
    unrm2 += blk.apply(vin, rs, a.m, a.n, tile * R, a.u, zacc, red, ush, stage);
  }
  if (threadIdx.x == 0) a.unrm2[blockIdx.x] = unrm2;
  store_partial<T, NS>(zacc, a.zpart, a.n, blockIdx.x, gridDim.x);
}

// z = sum of the partial vectors, in a fixed order; the workgroup that finishes last adds up
// the squared norm and derives the power of two that brings z back to unit magnitude.
struct ReduceArgs {
  const float* zpart;
  int parts, n;
  double* z;             // the sum ...
  float* z32;            // ... and the same rounded to float32, the next application's input
  double* normpart;      // one entry per workgroup
  double* nrm2;          // out: ||z||^2
  double* rescale;       // out: 2^-ilogb(||z||)
  unsigned* counter;     // zero before the launch; left at zero
};

__global__ __launch_bounds__(kReduceCols * kReduceGroups) void reduce_kernel(ReduceArgs a) {
  const int cl = threadIdx.x & (kReduceCols - 1), g = threadIdx.x / kReduceCols;
  const int col = blockIdx.x * kReduceCols + cl;
  __shared__ double red[kReduceGroups][kReduceCols];
  __shared__ bool last;
  // the block of this workgroup is contiguous: parts x kReduceCols floats
  const float* src = a.zpart + (int64_t)blockIdx.x * a.parts * kReduceCols + cl;
  double t = 0.0;
  for (int p0 = g; p0 < a.parts; p0 += 8 * kReduceGroups) {
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {   // all loads first: eight in flight per thread
      const int p = p0 + j * kReduceGroups;
      x[j] = p < a.parts ? src[(int64_t)p * kReduceCols] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) t += (double)x[j];
  }
  red[g][cl] = t;
  __syncthreads();
  if (threadIdx.x < kWave) {   // the first wave: four lanes per column, sixteen groups each
    const int quarter = threadIdx.x / kReduceCols;
    double zz = 0.0;
#pragma unroll
    for (int k = 0; k < kReduceGroups / 4; ++k) zz += red[quarter * (kReduceGroups / 4) + k][cl];
    zz += __shfl_xor(zz, 16);
    zz += __shfl_xor(zz, 32);
    if (threadIdx.x < kReduceCols && col < a.n) { a.z[col] = zz; a.z32[col] = (float)zz; }
    const double q = wave_sum((threadIdx.x < kReduceCols && col < a.n) ? zz * zz : 0.0);
    if (threadIdx.x == 0) {
      a.normpart[blockIdx.x] = q;
      __threadfence();
      last = atomicAdd(a.counter, 1u) == gridDim.x - 1;
    }
  }
  __syncthreads();
  if (last && threadIdx.x < kWave) {
    __threadfence();
    double q = 0.0;
    for (int k = threadIdx.x; k < (int)gridDim.x; k += kWave)
      q += __hip_atomic_load(a.normpart + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    q = wave_sum(q);
    if (threadIdx.x == 0) {
      *a.nrm2 = q;
      const double nz = sqrt(q);
      int e = (nz > 0.0 && nz < __builtin_inf()) ? ilogb(nz) : 0;
      e = e > 126 ? 126 : (e < -126 ? -126 : e);   // v = z * 2^-e is formed in float32
      *a.rescale = scalbn(1.0, -e);
      *a.counter = 0u;
    }
  }
}

// Stored triplet of one rank: U_1 = y/||y||, V_1 = p/||p|| in e4m3, sigma = ||p||/||y|| in
// fp16 (Algorithm 1), plus their decoded values for the deflation.
struct FinishArgs {
  const double* y; const double* ynrm2; int yparts; int m;
  const double* p; const double* pnrm2; int n;
  uint8_t* U; uint8_t* V; uint16_t* sigma16;
  double* ud; double* vd; double* sigma;
};

__global__ __launch_bounds__(256) void finish_kernel(FinishArgs a) {
  __shared__ double red[4];
  double t = 0.0;
  for (int k = threadIdx.x; k < a.yparts; k += 256) t += a.ynrm2[k];
  t = wave_sum(t);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = t;
  __syncthreads();
  const double ny = sqrt((red[0] + red[1]) + (red[2] + red[3]));
  const double np = sqrt(*a.pnrm2);
  const bool dead = !(ny > 0.0) || !(np > 0.0);
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < a.m) {
    const uint8_t c = dead ? 0 : e4m3_encode(a.y[i] / ny);
    a.U[i] = c;
    a.ud[i] = e4m3_decode(c);
  }
  if (i < a.n) {
    const uint8_t c = dead ? 0 : e4m3_encode(a.p[i] / np);
    a.V[i] = c;
    a.vd[i] = e4m3_decode(c);
  }
  if (i == 0) {
    const uint16_t h = dead ? 0 : fp16_encode_pos(np / ny);
    *a.sigma16 = h;
    *a.sigma = fp16_decode_pos(h);
  }
}

// ---- the whole loop in one launch, row blocks streamed -----------------------------------------
// All ranks and applications in one cooperative launch: the workgroups meet at a barrier
// between the steps that the separate kernels above end with, and stream their row blocks from
// memory in every application.  This is the form for matrices too large for the tile form
// further down (the MLP layers).
//
// The barrier is a counter in global memory that only grows.  A waiting workgroup gives up
// after spin_limit polls and raises `abort`, which makes every later wait return at once: the
// kernel always terminates, and the caller finds NaN in every sigma.
struct ChainArgs {
  float* A; int m, n;
  const float* S; int64_t lds; int r, it;
  uint8_t* U; uint8_t* V; uint16_t* sigma16;
  float* zpart; double* z; double* u; double* unrm2; double* normpart; double* ud; double* vd;
  float* zapp;          // one float32 copy of z per application, zstride floats apart
  int64_t zstride;
  double* sigma;        // the last rank's decoded sigma, for the residual kernel
  int* expo;            // r * (it + 1) entries preset to INT_MIN: largest exponent in each z
  unsigned* bar;        // kBarrierWords words preset to 0
  int* abort;           // preset to 0
  unsigned spin_limit;
};

template <int NS, int R>
__global__ __launch_bounds__(kChainThreads) void chain_kernel(ChainArgs a) {
  constexpr int T = kChainThreads;
  constexpr int kGroups = T / kReduceCols;   // 32 partial vectors in flight per column
  __shared__ double red[T / kWave * R];
  __shared__ double ush[R];
  __shared__ double sred[kGroups][kReduceCols];
  __shared__ float stage[T / kWave * 512];
  __shared__ double fin[T / kWave];
  const int tid = threadIdx.x, b = blockIdx.x, G = gridDim.x;
  const int m = a.m, n = a.n;
  const int tiles = (m + R - 1) / R;
  const int ncb = (n + kReduceCols - 1) / kReduceCols;
  unsigned phase = 0;
  int app = 0;
  double sg_prev = 0.0;

  for (int k = 0; k < a.r; ++k) {
    for (int i = 0; i <= a.it; ++i, ++app) {
      double zacc[NS][4];
#pragma unroll
      for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int c = 0; c < 4; ++c) zacc[s][c] = 0.0;
      double unrm2 = 0.0;
      float rs = 1.f;
      if (i > 0) {
        int e = __hip_atomic_load(a.expo + app - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        e = e == INT_MIN ? 0 : (e > 126 ? 126 : (e < -126 ? -126 : e));
        rs = scalbnf(1.f, -e);
      }
      // Every workgroup reads all of v.  Coherent loads of the same few lines from 256 places
      // are served one after the other by the memory side; ordinary loads are served by the L2
      // of each die after its first miss, and they are safe here because each application's z
      // has an address of its own that no cache can hold an older copy of.
      const float* v_in = i == 0 ? a.S + (int64_t)k * a.lds : a.zapp + (int64_t)(app - 1) * a.zstride;
      for (int tile = b; tile < tiles; tile += G) {
        const float* vin = v_in;
        const double* vd = a.vd;
        asm volatile("" : "+s"(vin), "+s"(vd));
        RowBlock<T, NS, R, true> blk;
        blk.load(a.A, m, n, tile * R, i == 0 && k > 0, sg_prev, a.ud, vd);
        unrm2 += blk.apply(vin, rs, m, n, tile * R, a.u, zacc, red, ush, stage);
      }
      store_partial<T, NS, true>(zacc, a.zpart, n, b, G);
      if (tid == 0) store_dev(a.unrm2 + b, unrm2);
      grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);

      // this workgroup's column blocks of z = sum of the partial vectors
      const bool last_app = i == a.it;
      for (int cb = b; cb < ncb; cb += G) {
        const int cl = tid & (kReduceCols - 1), g = tid / kReduceCols;
        const int col = cb * kReduceCols + cl;
        const float* src = a.zpart + (int64_t)cb * G * kReduceCols + cl;
        double t = 0.0;
        for (int p0 = g; p0 < G; p0 += 8 * kGroups) {
          float x[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int p = p0 + j * kGroups;
            x[j] = p < G ? load_dev(src + (int64_t)p * kReduceCols) : 0.f;
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) t += (double)x[j];
        }
        sred[g][cl] = t;
        __syncthreads();
        if (tid < kWave) {
          const int quarter = tid / kReduceCols;
          double zz = 0.0;
#pragma unroll
          for (int q = 0; q < kGroups / 4; ++q) zz += sred[quarter * (kGroups / 4) + q][cl];
          zz += __shfl_xor(zz, 16);
          zz += __shfl_xor(zz, 32);
          const bool mine = tid < kReduceCols && col < n;
          if (mine) {
            store_dev(a.zapp + (int64_t)app * a.zstride + col, (float)zz);
            a.z[col] = zz;   // read back by this workgroup only
          }
          if (!last_app) {
            int e = (mine && zz != 0.0 && fabs(zz) < __builtin_inf()) ? ilogb(zz) : INT_MIN;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) e = max(e, __shfl_xor(e, o));
            if (tid == 0 && e != INT_MIN) atomicMax(a.expo + app, e);
          } else {
            const double q2 = wave_sum(mine ? zz * zz : 0.0);
            if (tid == 0) store_dev(a.normpart + cb, q2);
          }
        }
        __syncthreads();
      }
      grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);
    }

    // the stored triplet of rank k: every workgroup derives the same norms and sigma, and
    // encodes the entries of U and V it produced itself
    const double ny = sqrt(block_sum<T>(a.unrm2, G, fin));
    const double np = sqrt(block_sum<T>(a.normpart, ncb, fin));
    const bool dead = !(ny > 0.0) || !(np > 0.0);
    const uint16_t h = dead ? 0 : fp16_encode_pos(np / ny);
    sg_prev = fp16_decode_pos(h);
    if (b == 0 && tid == 0) { a.sigma16[k] = h; *a.sigma = sg_prev; }
    for (int tile = b; tile < tiles; tile += G) {
      const int row = tile * R + tid;
      if (tid < R && row < m) {
        const uint8_t c = dead ? 0 : e4m3_encode(a.u[row] / ny);
        a.U[(int64_t)k * m + row] = c;
        store_dev(a.ud + row, e4m3_decode(c));
      }
    }
    for (int cb = b; cb < ncb; cb += G) {
      const int col = cb * kReduceCols + tid;
      if (tid < kReduceCols && col < n) {
        const uint8_t c = dead ? 0 : e4m3_encode(a.z[col] / np);
        a.V[(int64_t)k * n + col] = c;
        store_dev(a.vd + col, e4m3_decode(c));
      }
    }
    grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);
  }

  if (b == 0 && __hip_atomic_load(a.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
    for (int k = tid; k < a.r; k += T) a.sigma16[k] = 0x7e00;
}

// ---- the whole loop on a matrix that fits the registers of the chip ---------------------------
// When the matrix has at most 256 tiles of 256 x 256 (64 MB of float32: the attention
// projections of a 7B model), a workgroup keeps ONE TILE, not a block of rows, for the whole
// loop.  Tile (p, q) then exchanges 256 partial sums per product instead of a whole partial
// vector: its share of u = A v goes to the Q tiles of its row of tiles, its share of z = A^T u
// to the P tiles of its column, and each tile adds up the partial sums it needs itself.  So
// an application moves 1/8 of the data of the row-block form and has no separate summation
// step; only the norms of a rank's last vectors need everybody (once per rank).
//
// There is no barrier between the steps of an application.  Every exchanged number is an
// 8-byte word, the float in the low half and the number of the application in the high half,
// written with one device-coherent store; a reader loads the words it needs and loads them
// again until their high halves show the application it is waiting for.  Store, signal and
// load thus cost one trip to memory instead of three (wait for the store, arrive and poll,
// load).  A reader gives up after spin_limit rounds and raises `abort`, like the barriers.
//
// The power of two that keeps the vectors in range travels with the data: every tile attaches
// the largest exponent of its piece of v to its partial u; the tiles of a row of tiles see
// all pieces, take the maximum and scale u instead of v (the same thing, A being linear).
// Partial sums alternate between two buffers, so that a tile may write those of the next
// application while a slower tile of its group still reads the last ones: a tile writes
// application i + 2 only after it has seen application i + 1 from every tile of the group, and
// each of those published it after it had read application i.
constexpr int kTile = 256;
constexpr int kTilePart = kTile + 32;   // 256 partial sums and, in the next word, the exponent

struct TileArgs {
  float* A; int m, n;
  const float* S; int64_t lds; int r, it;
  uint8_t* U; uint8_t* V; uint16_t* sigma16;
  int P, Q;             // tiles down and across; the grid has P * Q workgroups
  unsigned long long* upart;   // [2][P][Q][kTilePart] tagged words, preset to 0 (tags start at 1)
  unsigned long long* zpart;   // [2][P][Q][kTilePart]
  double* normy;        // [2][P]: sum of squares of a rank's y by row of tiles
  double* normp;        // [2][Q]: the same for p by column of tiles
  double* ud; double* vd; double* sigma;   // the last rank's decoded triplet, for the residual kernel
  unsigned* bar;        // the two-level barrier of all workgroups
  int* abort;
  unsigned spin_limit;
};

// Sum of squares of an LDS array over the workgroup, fixed order; the same value in every thread.
template <int T>
__device__ __forceinline__ double block_sum_squares(const double* x, int count, double* scratch) {
  double t = 0.0;
  for (int j = threadIdx.x; j < count; j += T) t = fma(x[j], x[j], t);
  t = wave_sum(t);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = t;
  __syncthreads();
  double total = 0.0;
#pragma unroll
  for (int wv = 0; wv < T / kWave; ++wv) total += scratch[wv];
  return total;
}

// Entry (threadIdx.x & 255) of the sum of `count` partial vectors `stride` words apart, each word
// tagged `tag`, for a workgroup of 512 threads: each half of the workgroup takes every other
// vector, eight loads in flight per thread (one after the other they are a chain of trips to
// memory), repeated until all eight carry the tag; the two halves meet in `tmp` (2 x 256
// doubles).  Valid in threads 0..255 after the call.
__device__ __forceinline__ double sum_partials(const unsigned long long* base, int count, int64_t stride,
                                               unsigned tag, double* tmp, int* abort, unsigned spin_limit) {
  const int e = threadIdx.x & (kTile - 1), half = threadIdx.x >> 8;
  double t = 0.0;
  unsigned spins = 0;
  for (int j0 = half; j0 < count; j0 += 16) {
    unsigned long long x[8];
    bool ready;
    do {
      ready = true;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        x[k] = (unsigned long long)tag << 32;
        if (j0 + 2 * k < count) x[k] = load_tagged(base + (int64_t)(j0 + 2 * k) * stride + e);
        ready = ready && (unsigned)(x[k] >> 32) == tag;
      }
    } while (!ready && keep_waiting(spins, abort, spin_limit));
#pragma unroll
    for (int k = 0; k < 8; ++k) t += (double)__uint_as_float((unsigned)x[k]);
  }
  __syncthreads();
  tmp[half * kTile + e] = t;
  __syncthreads();
  return tmp[e] + tmp[kTile + e];
}

__global__ __launch_bounds__(512) void tile_chain_kernel(TileArgs a) {
  constexpr int T = 512, kWaves = T / kWave, kRowsPerWave = kTile / kWaves;   // 8 waves x 32 rows
  __shared__ double zsum[kTile];        // this column of tiles' piece of z (= v of the next application, p at the end)
  __shared__ float vsh[kTile];          // ... as the float32 vector the products use
  __shared__ double ush[kTile];         // this row of tiles' piece of u, scaled
  __shared__ float red2[kWaves][kTile];
  __shared__ float stage[kWaves * 512];   // per wave: 8 rows x 64 lanes on their way to the row sums
  __shared__ double udsh[kTile], vdsh[kTile];
  __shared__ double tmp[2 * kTile];
  __shared__ double fin[kWaves];
  __shared__ int esh[kWaves];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int m = a.m, n = a.n, P = a.P, Q = a.Q;
  const int p = blockIdx.x / Q, q = blockIdx.x - p * Q;
  const int row_base = p * kTile, col_base = q * kTile;
  const int my_row0 = row_base + w * kRowsPerWave;   // this wave's 32 rows
  const int my_col = col_base + lane * 4;            // this lane's 4 columns
  const int64_t part_stride = (int64_t)P * Q * kTilePart;

  float wt[kRowsPerWave][4];
#pragma unroll
  for (int i = 0; i < kRowsPerWave; ++i) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (my_row0 + i < m && my_col < n) v = *reinterpret_cast<const float4*>(a.A + (int64_t)(my_row0 + i) * n + my_col);
    wt[i][0] = v.x; wt[i][1] = v.y; wt[i][2] = v.z; wt[i][3] = v.w;
  }

  unsigned gphase = 0;
  int app = 0;
  for (int k = 0; k < a.r; ++k) {
    for (int i = 0; i <= a.it; ++i, ++app) {
      const int buf = app & 1;
      const unsigned tag = (unsigned)app + 1u;   // what this application writes; it reads z tagged `app`
      // ---- v for this column of tiles: the sketch vector, or the sum of the partial z of the tiles above and below
      int e_loc = INT_MIN;
      if (i == 0) {
        const int col = col_base + tid;
        if (tid < kTile) vsh[tid] = col < n ? a.S[(int64_t)k * a.lds + col] : 0.f;
      } else {
        const double t = sum_partials(a.zpart + (int64_t)(buf ^ 1) * part_stride + (int64_t)q * kTilePart, P,
                                      (int64_t)Q * kTilePart, (unsigned)app, tmp, a.abort, a.spin_limit);
        if (tid < kTile) {
          vsh[tid] = (float)t;
          if (t != 0.0 && fabs(t) < __builtin_inf()) e_loc = ilogb(t);
        }
      }
      if (i > 0) {   // largest exponent of the piece: wave maximum, then over the waves that hold data
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) e_loc = max(e_loc, __shfl_xor(e_loc, o));
        if (lane == 0) esh[w] = e_loc;
      }
      __syncthreads();
      if (i > 0) e_loc = max(max(esh[0], esh[1]), max(esh[2], esh[3]));

      // ---- this tile's share of u = A v: 32 rows per wave, reduced over the 64 lanes
      {
        const float4 v = *reinterpret_cast<const float4*>(&vsh[lane * 4]);
#pragma unroll
        for (int h = 0; h < kRowsPerWave / 8; ++h) {
          float us[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float* wr = wt[h * 8 + j];
            us[j] = fmaf(wr[3], v.w, fmaf(wr[2], v.z, fmaf(wr[1], v.y, wr[0] * v.x)));
          }
          const double t = wave_row_sums_staged(us, stage + w * 512);
          if ((lane & 7) == 0)
            store_tagged(a.upart + (int64_t)buf * part_stride + ((int64_t)p * Q + q) * kTilePart + w * kRowsPerWave +
                             h * 8 + (lane >> 3),
                         __float_as_uint((float)t), tag);
        }
        if (tid == 0)
          store_tagged(a.upart + (int64_t)buf * part_stride + ((int64_t)p * Q + q) * kTilePart + kTile,
                       (unsigned)e_loc, tag);
      }

      // ---- u for this row of tiles: the partial sums of the tiles to the left and right, scaled
      {
        const unsigned long long* row_parts = a.upart + (int64_t)buf * part_stride + (int64_t)p * Q * kTilePart;
        int e = INT_MIN;
        if (tid < Q) {
          unsigned spins = 0;
          unsigned long long hw;
          do hw = load_tagged(row_parts + (int64_t)tid * kTilePart + kTile);
          while ((unsigned)(hw >> 32) != tag && keep_waiting(spins, a.abort, a.spin_limit));
          e = (int)(unsigned)hw;
        }
        const double t = sum_partials(row_parts, Q, kTilePart, tag, tmp, a.abort, a.spin_limit);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) e = max(e, __shfl_xor(e, o));
        if (lane == 0) esh[w] = e;
        __syncthreads();
        e = max(max(esh[0], esh[1]), max(esh[2], esh[3]));   // Q <= 256: the first four waves
        if (tid < kTile) ush[tid] = t * unscale(e);
      }
      __syncthreads();

      // ---- this tile's share of z = A^T u: 4 columns per lane, reduced over the 8 waves
      {
        float zs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < kRowsPerWave; ++j) {
          const float uf = (float)ush[w * kRowsPerWave + j];
#pragma unroll
          for (int c = 0; c < 4; ++c) zs[c] = fmaf(wt[j][c], uf, zs[c]);
        }
        *reinterpret_cast<float4*>(&red2[w][lane * 4]) = make_float4(zs[0], zs[1], zs[2], zs[3]);
      }
      __syncthreads();
      if (tid < kTile) {
        double t = 0.0;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) t += (double)red2[wv][tid];
        store_tagged(a.zpart + (int64_t)buf * part_stride + ((int64_t)p * Q + q) * kTilePart + tid,
                     __float_as_uint((float)t), tag);
      }
    }

    // ---- the stored triplet of rank k.  y is ush (every tile of the row of tiles has it), p is the sum of the last
    // partial z of this column of tiles; their norms need all rows resp. columns of tiles.
    const int last = (app - 1) & 1, nb = k & 1;
    {
      const double t = sum_partials(a.zpart + (int64_t)last * part_stride + (int64_t)q * kTilePart, P,
                                    (int64_t)Q * kTilePart, (unsigned)app, tmp, a.abort, a.spin_limit);
      if (tid < kTile) zsum[tid] = t;
    }
    __syncthreads();
    const double y2 = block_sum_squares<T>(ush, kTile, fin);     // rows and columns outside the matrix hold zeros
    const double p2 = block_sum_squares<T>(zsum, kTile, fin);
    if (tid == 0) {
      if (q == 0) store_dev(a.normy + nb * P + p, y2);
      if (p == 0) store_dev(a.normp + nb * Q + q, p2);
    }
    grid_barrier(a.bar, ++gphase, a.abort, a.spin_limit);
    const double ny = sqrt(block_sum<T>(a.normy + nb * P, P, fin));
    const double np = sqrt(block_sum<T>(a.normp + nb * Q, Q, fin));
    const bool dead = !(ny > 0.0) || !(np > 0.0);
    const uint16_t h = dead ? 0 : fp16_encode_pos(np / ny);
    const double sg = fp16_decode_pos(h);
    if (blockIdx.x == 0 && tid == 0) { a.sigma16[k] = h; *a.sigma = sg; }
    if (tid < kTile) {
      const int row = row_base + tid, col = col_base + tid;
      const uint8_t cu = dead ? 0 : e4m3_encode(ush[tid] / ny);
      const uint8_t cv = dead ? 0 : e4m3_encode(zsum[tid] / np);
      udsh[tid] = e4m3_decode(cu);
      vdsh[tid] = e4m3_decode(cv);
      if (q == 0 && row < m) { a.U[(int64_t)k * m + row] = cu; a.ud[row] = udsh[tid]; }
      if (p == 0 && col < n) { a.V[(int64_t)k * n + col] = cv; a.vd[col] = vdsh[tid]; }
    }
    __syncthreads();
    // the deflation by this rank, in registers (the last rank's is left to the residual kernel)
    if (k + 1 < a.r) {
      double dv[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) dv[c] = sg * vdsh[lane * 4 + c];
#pragma unroll
      for (int j = 0; j < kRowsPerWave; ++j) {
        const double uj = udsh[w * kRowsPerWave + j];
#pragma unroll
        for (int c = 0; c < 4; ++c) wt[j][c] = (float)((double)wt[j][c] - uj * dv[c]);
      }
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < kRowsPerWave; ++i)
    if (my_row0 + i < m && my_col < n)
      *reinterpret_cast<float4*>(a.A + (int64_t)(my_row0 + i) * n + my_col) =
          make_float4(wt[i][0], wt[i][1], wt[i][2], wt[i][3]);
  if (blockIdx.x == 0 && __hip_atomic_load(a.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
    for (int k = tid; k < a.r; k += T) a.sigma16[k] = 0x7e00;
}

// R = (A - sigma u v^T) diag(s)^-1: the last rank's deflation and the way back from the scaled
// matrix (Algorithm 1).
__global__ __launch_bounds__(256) void residual_kernel(const float* __restrict__ A, int m, int n,
                                                       const double* __restrict__ sigma,
                                                       const double* __restrict__ ud, const double* __restrict__ vd,
                                                       const double* __restrict__ s, float* __restrict__ Rout,
                                                       int64_t ldr) {
  const int nb = (n + 1023) / 1024;
  const int c = ((int)(blockIdx.x % nb) * 256 + threadIdx.x) * 4;
  const int row = blockIdx.x / nb;
  if (c >= n) return;
  const float4 q = *reinterpret_cast<const float4*>(A + (int64_t)row * n + c);
  const double su = sigma ? *sigma * ud[row] : 0.0;
  const float in[4] = {q.x, q.y, q.z, q.w};
  float o[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const double v = sigma ? (double)in[k] - su * vd[c + k] : (double)in[k];
    o[k] = (float)(v / s[c + k]);
  }
  *reinterpret_cast<float4*>(Rout + (int64_t)row * ldr + c) = make_float4(o[0], o[1], o[2], o[3]);
}

// ---- host side -----------------------------------------------------------------------------------
// rows per workgroup by number of column sweeps (registers: 4 * sweeps * rows floats per thread)
// Shape of a pass by number of columns: 512 threads and one workgroup per compute unit, which
// gives a thread 256 registers; they hold 4 * sweeps * rows floats of A, 4 * sweeps float64
// sums of z and `rows` float64 sums of u.
constexpr int kPassThreads = 512;
struct PassShape { int ns, rows; };
inline PassShape pass_shape(int64_t n) {
  if (n <= 2048) return {1, 16};
  if (n <= 4096) return {2, 16};
  if (n <= 8192) return {4, 8};
  if (n <= 12288) return {6, 4};
  if (n <= 16384) return {8, 2};
  return {16, 1};
}

// workspace of the tile form: tagged partial sums (two buffers each) and norms
constexpr size_t kTilePartBytes = (size_t)2 * kComputeUnits * kTilePart * sizeof(unsigned long long);
constexpr size_t kTileNormBytes = (size_t)2 * kComputeUnits * sizeof(double);
constexpr size_t kTileWorkspaceBytes = 2 * kTilePartBytes + 2 * kTileNormBytes;

constexpr int kMaxChainApps = 16384;   // applications (rank x iteration) one cooperative launch can hold
constexpr size_t kChainVectorBytes = size_t{16} << 20;   // room for their float32 copies of z

struct Layout {
  size_t A, zpart, z, z32, u, unrm2, normpart, ud, vd, scalars, barrier, expo, zapp, tile, sf, shares, resident, total;
  int parts;    // workgroups of a pass when every step is a launch of its own
  int groups;   // workgroups of the single cooperative launch
};
inline Layout layout(int64_t m, int64_t n) {
  Layout L{};
  const PassShape ps = pass_shape(n);
  const int64_t tiles = ceil_div(m, ps.rows);
  L.parts = (int)(tiles < kComputeUnits ? tiles : kComputeUnits);
  const int64_t want = tiles > ceil_div(n, kReduceCols) ? tiles : ceil_div(n, kReduceCols);
  L.groups = (int)(want < kComputeUnits ? want : kComputeUnits);
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
  L.A = take((size_t)m * n * sizeof(float));
  L.zpart = take((size_t)ceil_div(n, kReduceCols) * kComputeUnits * kReduceCols * sizeof(float));
  L.z = take((size_t)n * sizeof(double));
  L.z32 = take((size_t)n * sizeof(float));
  L.u = take((size_t)m * sizeof(double));
  L.unrm2 = take((size_t)kComputeUnits * sizeof(double));
  L.normpart = take((size_t)kMaxNormParts * sizeof(double));
  L.ud = take((size_t)m * sizeof(double));
  L.vd = take((size_t)n * sizeof(double));
  L.scalars = take(256);
  L.barrier = take((size_t)kBarrierWords * sizeof(unsigned));
  L.expo = take((size_t)kMaxChainApps * sizeof(int));
  L.zapp = take(kChainVectorBytes);
  L.tile = take(kTileWorkspaceBytes);
  L.sf = take((size_t)n * sizeof(float));
  L.shares = take((size_t)2 * kMaxStreamRank * kComputeUnits * sizeof(double));
  L.resident = take(kResidentWorkspaceBytes);
  L.total = o;
  return L;
}

template <int NS, int R>
void launch_pass(const PassArgs& a, int parts, hipStream_t st) {
  if (a.sigma)
    pass_kernel<kPassThreads, NS, R, true><<<(unsigned)parts, kPassThreads, 0, st>>>(a);
  else
    pass_kernel<kPassThreads, NS, R, false><<<(unsigned)parts, kPassThreads, 0, st>>>(a);
}

// Whether `groups` workgroups of the chain kernel can be resident at once on the current device.
template <int NS, int R>
bool chain_fits(int groups) {
  int dev = 0, coop = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, chain_kernel<NS, R>, kChainThreads, 0) != hipSuccess)
    return false;
  return (int64_t)per_cu * cus >= groups;
}

template <int NS, int R>
bool launch_chain(ChainArgs& a, int groups, hipStream_t st) {
  if (!chain_fits<NS, R>(groups)) return false;
  void* params[] = {&a};
  if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(chain_kernel<NS, R>), dim3((unsigned)groups),
                                 dim3(kChainThreads), params, 0, st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

bool launch_tile_chain(TileArgs& a, hipStream_t st) {
  int dev = 0, coop = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tile_chain_kernel, 512, 0) != hipSuccess) return false;
  if ((int64_t)per_cu * cus < (int64_t)a.P * a.Q) return false;
  void* params[] = {&a};
  if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(tile_chain_kernel), dim3((unsigned)(a.P * a.Q)),
                                 dim3(512), params, 0, st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

}  // namespace

size_t abs_sum_workspace_bytes(int64_t n) { return align_up((size_t)kAbsSlices * n * sizeof(double), 256); }

ptq_status abs_sum_launch(double* asum, const void* X, ptq_dtype xdt, int64_t t, int64_t n, int64_t ldx, void* ws,
                          hipStream_t st) {
  double* partial = static_cast<double*>(ws);
  dim3 g((unsigned)ceil_div(n, kAbsCols), kAbsSlices);
  if (xdt == PTQ_BF16)
    abs_sum_kernel<PTQ_BF16><<<g, 256, 0, st>>>(X, ldx, t, (int)n, partial);
  else
    abs_sum_kernel<PTQ_F32><<<g, 256, 0, st>>>(X, ldx, t, (int)n, partial);
  abs_sum_finish_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(partial, (int)n, asum);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status activation_scale_launch(const double* asum, int64_t tokens, int64_t n, double* s, hipStream_t st) {
  scale_kernel<<<1, 1024, 0, st>>>(asum, (double)tokens, (int)n, s);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

// Process-wide selection for the library's own tests and comparisons (not part of the documented
// interface): 0 = the form the shapes call for, 1 = resident, 2 = stream, 3 = row blocks of the float32
// running matrix, 4 = one launch per step; and the number of rounds a waiting workgroup spins.
static std::atomic<int> g_launch_form{0};
static std::atomic<unsigned> g_spin_limit{1u << 21};
void r1svd_select(int launch_form, long long spin_limit) {
  g_launch_form.store(launch_form >= 0 && launch_form <= 4 ? launch_form : 0, std::memory_order_relaxed);
  g_spin_limit.store(spin_limit < 0 ? (1u << 21) : (unsigned)spin_limit, std::memory_order_relaxed);
}

size_t r1svd_workspace_bytes(int64_t m, int64_t n) { return layout(m, n).total; }
int64_t r1svd_max_columns() { return kMaxColumns; }

ptq_status r1svd_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* s,
                        const float* S, int64_t lds, int r, int it, uint8_t* U, uint8_t* V, uint16_t* sigma16,
                        float* Rout, int64_t ldr, void* ws, hipStream_t st) {
  const Layout L = layout(m, n);
  const PassShape ps = pass_shape(n);
  char* base = static_cast<char*>(ws);
  float* A = reinterpret_cast<float*>(base + L.A);
  float* zpart = reinterpret_cast<float*>(base + L.zpart);
  double* z = reinterpret_cast<double*>(base + L.z);
  float* z32 = reinterpret_cast<float*>(base + L.z32);
  double* u = reinterpret_cast<double*>(base + L.u);
  double* unrm2 = reinterpret_cast<double*>(base + L.unrm2);
  double* normpart = reinterpret_cast<double*>(base + L.normpart);
  double* ud = reinterpret_cast<double*>(base + L.ud);
  double* vd = reinterpret_cast<double*>(base + L.vd);
  double* scal = reinterpret_cast<double*>(base + L.scalars);   // [0] ||z||^2  [1] rescale  [2] sigma
  unsigned* counter = reinterpret_cast<unsigned*>(scal + 3);
  clear_counter_kernel<<<1, kWave, 0, st>>>(counter);   // a kernel, so that the call can be captured in a graph

  // rounds a workgroup waits for another before it gives up, and the form of the loop: one cooperative
  // launch for the whole loop where the device can hold it, in the form the shapes call for, unless
  // the library's own tests have selected another one (r1svd_select below)
  const unsigned spin_limit = g_spin_limit.load(std::memory_order_relaxed);
  const int mode = g_launch_form.load(std::memory_order_relaxed);
  const auto mode_is = [&](const char* name) {
    return (mode == 1 && std::strcmp(name, "resident") == 0) || (mode == 2 && std::strcmp(name, "stream") == 0) ||
           (mode == 3 && std::strcmp(name, "rows") == 0) || (mode == 4 && std::strcmp(name, "steps") == 0);
  };
  const int64_t TP = ceil_div(m, kTile), TQ = ceil_div(n, kTile);
  const bool tile_form = r > 0 && TP * TQ <= kComputeUnits && !mode_is("steps") && !mode_is("rows") &&
                         !mode_is("stream") && !mode_is("resident");
  const int64_t zstride = (int64_t)align_up((size_t)n * sizeof(float), 256) / (int64_t)sizeof(float);
  const bool one_launch_holds = r > 0 && (int64_t)r * (it + 1) <= kMaxChainApps &&
                                (size_t)r * (it + 1) * zstride * sizeof(float) <= kChainVectorBytes;
  int* abort_flag = reinterpret_cast<int*>(counter + 1);
  unsigned* bar = reinterpret_cast<unsigned*>(base + L.barrier);

  // A bfloat16 weight too large for the tile form is used as it is, never copied or rewritten: kept
  // on the chip if it fits there (resident form), else streamed in every application.
  if (wdt == PTQ_BF16 && !tile_form && !mode_is("steps") && !mode_is("rows") && one_launch_holds &&
      r <= kMaxStreamRank && n <= kMaxStreamColumns && n % 8 == 0 && ldw % 8 == 0 &&
      reinterpret_cast<uintptr_t>(W) % 16 == 0) {
    const R1svdBf16Call call{static_cast<const uint16_t*>(W), ldw, m, n, s, S, lds, r, it, U, V, sigma16, Rout, ldr,
                             reinterpret_cast<float*>(base + L.sf), reinterpret_cast<double*>(base + L.shares),
                             reinterpret_cast<int*>(base + L.expo), bar, abort_flag, zpart, z, u, unrm2, normpart,
                             reinterpret_cast<float*>(base + L.zapp), zstride, base + L.resident, spin_limit,
                             mode_is("stream")};
    if (r1svd_bf16_launch(call, st)) {
      PTQ_HIP_CHECK_LAUNCH();
      return PTQ_OK;
    }
  }

  const unsigned ge = (unsigned)(ceil_div(n, 1024) * m);   // one workgroup per 1024 columns of a row
  switch (wdt) {
    case PTQ_F32: scale_weight_kernel<PTQ_F32><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    case PTQ_BF16: scale_weight_kernel<PTQ_BF16><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    case PTQ_F64: scale_weight_kernel<PTQ_F64><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    default: return PTQ_ERR_DTYPE;
  }

  bool chained = false;
  // a matrix of at most 256 tiles stays in registers, a tile per workgroup
  if (tile_form) {
    char* tw = base + L.tile;
    unsigned long long* upart = reinterpret_cast<unsigned long long*>(tw);
    unsigned long long* zp2 = reinterpret_cast<unsigned long long*>(tw + kTilePartBytes);
    double* normy = reinterpret_cast<double*>(tw + 2 * kTilePartBytes);
    double* normp = reinterpret_cast<double*>(tw + 2 * kTilePartBytes + kTileNormBytes);
    // tags of an earlier call must not be mistaken for this one's: the tagged words start at zero
    const int words = (int)(2 * kTilePartBytes / sizeof(unsigned));
    tile_init_kernel<<<(unsigned)ceil_div(words, 256), 256, 0, st>>>(reinterpret_cast<unsigned*>(tw), words, abort_flag);
    tile_init_kernel<<<(unsigned)ceil_div(kBarrierWords, 256), 256, 0, st>>>(bar, kBarrierWords, abort_flag);
    TileArgs ta{A, (int)m, (int)n, S, lds, r, it, U, V, sigma16, (int)TP, (int)TQ, upart, zp2, normy, normp,
                ud, vd, scal + 2, bar, abort_flag, spin_limit};
    chained = launch_tile_chain(ta, st);
  }
  if (!chained && one_launch_holds && !mode_is("steps")) {
    int* expo = reinterpret_cast<int*>(base + L.expo);
    const int apps = r * (it + 1);
    const int init = apps > kBarrierWords ? apps : kBarrierWords;
    chain_init_kernel<<<(unsigned)ceil_div(init, 256), 256, 0, st>>>(expo, apps, bar, abort_flag);
    ChainArgs ca{A, (int)m, (int)n, S, lds, r, it, U, V, sigma16, zpart, z, u, unrm2, normpart, ud, vd,
                 reinterpret_cast<float*>(base + L.zapp), zstride, scal + 2, expo, bar, abort_flag, spin_limit};
    switch (ps.ns) {
      case 1: chained = launch_chain<1, 16>(ca, L.groups, st); break;
      case 2: chained = launch_chain<2, 16>(ca, L.groups, st); break;
      case 4: chained = launch_chain<4, 8>(ca, L.groups, st); break;
      case 6: chained = launch_chain<6, 4>(ca, L.groups, st); break;
      case 8: chained = launch_chain<8, 2>(ca, L.groups, st); break;
      default: chained = launch_chain<16, 1>(ca, L.groups, st); break;
    }
    if (!chained) clear_counter_kernel<<<1, kWave, 0, st>>>(counter);
  }

  const unsigned reduce_grid = (unsigned)ceil_div(n, kReduceCols);
  for (int k = 0; k < r && !chained; ++k) {
    for (int i = 0; i <= it; ++i) {
      PassArgs pa{A, (int)m, (int)n, i == 0 ? S + (int64_t)k * lds : z32, i == 0 ? nullptr : scal + 1,
                  u, unrm2, zpart, (i == 0 && k > 0) ? scal + 2 : nullptr, ud, vd};
      switch (ps.ns) {
        case 1: launch_pass<1, 16>(pa, L.parts, st); break;
        case 2: launch_pass<2, 16>(pa, L.parts, st); break;
        case 4: launch_pass<4, 8>(pa, L.parts, st); break;
        case 6: launch_pass<6, 4>(pa, L.parts, st); break;
        case 8: launch_pass<8, 2>(pa, L.parts, st); break;
        default: launch_pass<16, 1>(pa, L.parts, st); break;
      }
      ReduceArgs ra{zpart, L.parts, (int)n, z, z32, normpart, scal, scal + 1, counter};
      reduce_kernel<<<reduce_grid, kReduceCols * kReduceGroups, 0, st>>>(ra);
    }
    FinishArgs fa{u, unrm2, L.parts, (int)m, z, scal, (int)n, U + (int64_t)k * m, V + (int64_t)k * n,
                  sigma16 + k, ud, vd, scal + 2};
    finish_kernel<<<(unsigned)ceil_div(m > n ? m : n, 256), 256, 0, st>>>(fa);
    PTQ_HIP_CHECK_LAUNCH();
  }
  residual_kernel<<<ge, 256, 0, st>>>(A, (int)m, (int)n, r > 0 ? scal + 2 : nullptr, ud, vd, s, Rout, ldr);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq

