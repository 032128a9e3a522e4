// Scaled rank-one randomized sketching (paper Sec. 3.3, Eq. 9-11; Algorithm 1, inner loop)
// and the activation scale that precedes it.
//
// One rank costs  y = (A A^T)^it A v,  p = A^T y.  Written as  y = A (A^T A)^it v  this is
// it + 1 applications of "u = A v, z = A^T u" to the same matrix, and both products of one
// application can be taken from ONE pass over A: a workgroup owns a block of R complete rows,
// keeps them in registers, finishes its R entries of u = A v (a reduction inside the
// workgroup), and then multiplies the same registers by those entries to get its share of
// z = A^T u, which it writes as a partial vector.  A second small kernel adds the partial
// vectors in a fixed order.  So a rank reads A  it + 1  times instead of  2 it + 2  times,
// every sum has a fixed order (results are reproducible), and the chain is bound by the rate
// at which A (float32, rewritten once per rank by the deflation) streams from memory.
//
// Arithmetic: A is stored in float32; every product and sum is float64.  Vectors grow by
// sigma_1^2 per application; they are rescaled by a power of two (exact) taken from the norm
// of the previous result, so the printed formula is evaluated as it stands.
#include "common.h"

namespace ptq {
namespace {

constexpr int kComputeUnits = 256;
constexpr int kMaxColumns = 32768;
constexpr int kReduceCols = 16;                   // columns per workgroup of the partial-vector sum
constexpr int kReduceGroups = 64;                 // partial vectors in flight per column
constexpr int kMaxNormParts = kMaxColumns / kReduceCols;
static_assert(kReduceCols * 4 == kWave, "the last step of the sum pairs four lanes per column");

// ---- small floating point formats --------------------------------------------------------
// Nearest value with MANT explicit mantissa bits and smallest normal exponent EMIN, ties to
// even, as the integer  (biased exponent << MANT) + mantissa  (subnormals: the bare mantissa);
// the caller adds the sign and handles overflow.  Exact: only scalings by powers of two and
// one rint.
template <int MANT, int EMIN>
__device__ __forceinline__ int small_float_code(double a) {
  if (a == 0.0) return 0;
  int e = ilogb(a);
  e = e < EMIN ? EMIN : e;
  const double r = rint(scalbn(a, MANT - e));     // in [0, 2^(MANT+1)]
  return ((e - EMIN) << MANT) + (int)r;
}

// e4m3: 4 exponent bits (bias 7), 3 mantissa bits, subnormals, largest finite value 448,
// no infinities; saturating.
__device__ __forceinline__ uint8_t e4m3_encode(double x) {
  const double a = fabs(x);
  int code;
  if (!(a == a)) code = 0x7f;
  else if (a >= 448.0) code = 0x7e;
  else { code = small_float_code<3, -6>(a); code = code > 0x7e ? 0x7e : code; }
  return (uint8_t)(code | (signbit(x) ? 0x80 : 0));
}
__device__ __forceinline__ double e4m3_decode(uint8_t c) {
  const int ef = (c >> 3) & 0xf, mt = c & 7;
  const double mag = ef == 0 ? scalbn((double)mt, -9) : scalbn((double)(8 + mt), ef - 10);
  return (c & 0x80) ? -mag : mag;
}
// IEEE binary16 bits of a non-negative double (overflow gives infinity).
__device__ __forceinline__ uint16_t fp16_encode_pos(double a) {
  if (!(a == a)) return 0x7e00;
  if (a >= 65520.0) return 0x7c00;
  return (uint16_t)small_float_code<10, -14>(a);
}
__device__ __forceinline__ double fp16_decode_pos(uint16_t h) {
  const int ef = h >> 10, mt = h & 0x3ff;
  if (ef == 31) return mt ? __builtin_nan("") : __builtin_inf();
  return ef == 0 ? scalbn((double)mt, -24) : scalbn((double)(1024 + mt), ef - 25);
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

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
  const float* vin32;       // first application of a rank: the sketch vector ...
  const double* vin;        // ... afterwards the previous z
  const double* rescale;    // power of two applied to vin (null: 1)
  double* u;                // m
  double* unrm2;            // per workgroup: sum of squares of its entries of u
  double* zpart;            // one partial z per workgroup, see the end of the kernel for the layout
  // deflation by the previous rank's stored triplet, applied to A while it is loaded
  const double* sigma;      // null: none
  const double* ud;         // m
  const double* vd;         // n
};

// T threads; a thread owns 4 adjacent columns in each of NS sweeps of 4 T columns; R rows per block.
template <int T, int NS, int R, bool DEFLATE>
__global__ __launch_bounds__(T, (T == 512 && NS <= 2) ? 4 : 2) void pass_kernel(PassArgs a) {
  constexpr int kPassThreads = T, kPassWaves = T / kWave;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = a.n;
  __shared__ double red[kPassWaves][R];
  __shared__ double ush[R];

  double zacc[NS][4];
#pragma unroll
  for (int s = 0; s < NS; ++s)
#pragma unroll
    for (int c = 0; c < 4; ++c) zacc[s][c] = 0.0;
  double unrm2 = 0.0;   // thread 0 only
  const double rs = a.rescale ? *a.rescale : 1.0;
  const int tiles = (a.m + R - 1) / R;

  // a workgroup walks over row blocks and keeps adding to the same partial z, so that the
  // number of partial vectors is the number of workgroups, whatever the number of rows
  for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int row0 = tile * R;
    // the vectors are re-read (from cache) for every row block: kept in registers across the
    // loop they would take 8 per sweep and push the block's own data out
    const double* vin = a.vin;
    const float* vin32 = a.vin32;
    const double* vd = a.vd;
    asm volatile("" : "+s"(vin), "+s"(vin32), "+s"(vd));
    float w[NS][R][4];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 4 * (tid + kPassThreads * s);
      double dv[4] = {0.0, 0.0, 0.0, 0.0};
      if (DEFLATE && col < n) {
        const double sg = *a.sigma;
#pragma unroll
        for (int c = 0; c < 4; ++c) dv[c] = sg * vd[col + c];
      }
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const int row = row0 + i;
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col < n && row < a.m) {
          float4* p = reinterpret_cast<float4*>(a.A + (int64_t)row * n + col);
          q = *p;
          if (DEFLATE) {
            const double ui = a.ud[row];
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

    // u = A v for the R rows of this block
    double us[R];
#pragma unroll
    for (int i = 0; i < R; ++i) us[i] = 0.0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 4 * (tid + kPassThreads * s);
      double v[4] = {0.0, 0.0, 0.0, 0.0};
      if (col < n) {
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] = (vin32 ? (double)vin32[col + c] : vin[col + c]) * rs;
      }
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) us[i] = fma((double)w[s][i][c], v[c], us[i]);
    }
    // R sums over the 64 lanes at once: each exchange halves the number of values a lane
    // carries (the lane keeps the rows its bit selects and hands over the others), so R = 16
    // takes 8 + 4 + 2 + 1 exchanges and two plain ones instead of 16 x 6
    {
      int width = 32;
#pragma unroll
      for (int cnt = R; cnt > 1; cnt >>= 1, width >>= 1) {
        const bool upper = (lane & width) != 0;
#pragma unroll
        for (int j = 0; j < cnt / 2; ++j) {
          const double send = upper ? us[j] : us[j + cnt / 2];
          const double keep = upper ? us[j + cnt / 2] : us[j];
          us[j] = keep + __shfl_xor(send, width);
        }
      }
#pragma unroll
      for (; width >= 1; width >>= 1) us[0] += __shfl_xor(us[0], width);
      constexpr int kLanesPerRow = kWave / R;
      if ((lane & (kLanesPerRow - 1)) == 0) red[wave][lane / kLanesPerRow] = us[0];
    }
    __syncthreads();
    if (tid < R) {
      double t = 0.0;
#pragma unroll
      for (int wv = 0; wv < kPassWaves; ++wv) t += red[wv][tid];
      ush[tid] = t;
      if (row0 + tid < a.m) a.u[row0 + tid] = t;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
      for (int i = 0; i < R; ++i) unrm2 = fma(ush[i], ush[i], unrm2);
    }

    // (the float32 values are what stays in registers between the two products: without this
    // the compiler keeps their float64 conversions alive instead and spills)
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) asm volatile("" : "+v"(w[s][i][c]));

    // this block's share of z = A^T u
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int i = 0; i < R; ++i) {
        const double ui = ush[i];
#pragma unroll
        for (int c = 0; c < 4; ++c) zacc[s][c] = fma((double)w[s][i][c], ui, zacc[s][c]);
      }
  }

  if (tid == 0) a.unrm2[blockIdx.x] = unrm2;
  // partial vectors are stored in blocks of kReduceCols columns, [column block][workgroup][column],
  // so that the sum over workgroups reads contiguous memory
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int col = 4 * (tid + kPassThreads * s);
    if (col < n) {
      double* o = a.zpart + ((int64_t)(col / kReduceCols) * gridDim.x + blockIdx.x) * kReduceCols + col % kReduceCols;
      *reinterpret_cast<double2*>(o) = make_double2(zacc[s][0], zacc[s][1]);
      *reinterpret_cast<double2*>(o + 2) = make_double2(zacc[s][2], zacc[s][3]);
    }
  }
}

// z = sum of the partial vectors, in a fixed order; the workgroup that finishes last adds up
// the squared norm and derives the power of two that brings z back to unit magnitude.
struct ReduceArgs {
  const double* zpart;
  int parts, n;
  double* z;
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
  // the block of this workgroup is contiguous: parts x kReduceCols doubles
  const double* src = a.zpart + (int64_t)blockIdx.x * a.parts * kReduceCols + cl;
  double t = 0.0;
  for (int p0 = g; p0 < a.parts; p0 += 8 * kReduceGroups) {
    double x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {   // all loads first: eight in flight per thread
      const int p = p0 + j * kReduceGroups;
      x[j] = p < a.parts ? src[(int64_t)p * kReduceCols] : 0.0;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) t += x[j];
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
    if (threadIdx.x < kReduceCols && col < a.n) a.z[col] = zz;
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
      *a.rescale = (nz > 0.0 && nz < __builtin_inf()) ? scalbn(1.0, -ilogb(nz)) : 1.0;
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
// Shape of a pass by number of columns.  The registers of a thread hold 4 * sweeps * rows
// floats of A plus 4 * sweeps float64 sums.  Up to 4096 columns two workgroups share a compute
// unit, so that one loads while the other computes; beyond that one workgroup takes all registers.
struct PassShape { int threads, ns, rows, groups; };
inline PassShape pass_shape(int64_t n) {
  if (n <= 2048) return {512, 1, 16, 2 * kComputeUnits};
  if (n <= 4096) return {512, 2, 8, 2 * kComputeUnits};
  if (n <= 8192) return {512, 4, 4, kComputeUnits};
  if (n <= 12288) return {512, 6, 2, kComputeUnits};
  if (n <= 16384) return {512, 8, 1, kComputeUnits};
  return {512, 16, 1, kComputeUnits};
}

struct Layout {
  size_t A, zpart, z, u, unrm2, normpart, ud, vd, scalars, total;
  int parts;
};
inline Layout layout(int64_t m, int64_t n) {
  Layout L{};
  const PassShape ps = pass_shape(n);
  const int64_t tiles = ceil_div(m, ps.rows);
  L.parts = (int)(tiles < ps.groups ? tiles : ps.groups);
  size_t o = 0;
  auto take = [&](size_t bytes) { const size_t at = o; o += align_up(bytes, 256); return at; };
  L.A = take((size_t)m * n * sizeof(float));
  L.zpart = take((size_t)ceil_div(n, kReduceCols) * L.parts * kReduceCols * sizeof(double));
  L.z = take((size_t)n * sizeof(double));
  L.u = take((size_t)m * sizeof(double));
  L.unrm2 = take((size_t)L.parts * sizeof(double));
  L.normpart = take((size_t)kMaxNormParts * sizeof(double));
  L.ud = take((size_t)m * sizeof(double));
  L.vd = take((size_t)n * sizeof(double));
  L.scalars = take(256);
  L.total = o;
  return L;
}

template <int T, int NS, int R>
void launch_pass(const PassArgs& a, int parts, hipStream_t st) {
  if (a.sigma)
    pass_kernel<T, NS, R, true><<<(unsigned)parts, T, 0, st>>>(a);
  else
    pass_kernel<T, NS, R, false><<<(unsigned)parts, T, 0, st>>>(a);
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

size_t r1svd_workspace_bytes(int64_t m, int64_t n) { return layout(m, n).total; }
int64_t r1svd_max_columns() { return kMaxColumns; }

ptq_status r1svd_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* s,
                        const float* S, int64_t lds, int r, int it, uint8_t* U, uint8_t* V, uint16_t* sigma16,
                        float* Rout, int64_t ldr, void* ws, hipStream_t st) {
  const Layout L = layout(m, n);
  const PassShape ps = pass_shape(n);
  char* base = static_cast<char*>(ws);
  float* A = reinterpret_cast<float*>(base + L.A);
  double* zpart = reinterpret_cast<double*>(base + L.zpart);
  double* z = reinterpret_cast<double*>(base + L.z);
  double* u = reinterpret_cast<double*>(base + L.u);
  double* unrm2 = reinterpret_cast<double*>(base + L.unrm2);
  double* normpart = reinterpret_cast<double*>(base + L.normpart);
  double* ud = reinterpret_cast<double*>(base + L.ud);
  double* vd = reinterpret_cast<double*>(base + L.vd);
  double* scal = reinterpret_cast<double*>(base + L.scalars);   // [0] ||z||^2  [1] rescale  [2] sigma
  unsigned* counter = reinterpret_cast<unsigned*>(scal + 3);
  clear_counter_kernel<<<1, kWave, 0, st>>>(counter);   // a kernel, so that the call can be captured in a graph

  const unsigned ge = (unsigned)(ceil_div(n, 1024) * m);   // one workgroup per 1024 columns of a row
  switch (wdt) {
    case PTQ_F32: scale_weight_kernel<PTQ_F32><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    case PTQ_BF16: scale_weight_kernel<PTQ_BF16><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    case PTQ_F64: scale_weight_kernel<PTQ_F64><<<ge, 256, 0, st>>>(W, ldw, (int)m, (int)n, s, A); break;
    default: return PTQ_ERR_DTYPE;
  }

  const unsigned reduce_grid = (unsigned)ceil_div(n, kReduceCols);
  for (int k = 0; k < r; ++k) {
    for (int i = 0; i <= it; ++i) {
      PassArgs pa{A, (int)m, (int)n, i == 0 ? S + (int64_t)k * lds : nullptr, z, i == 0 ? nullptr : scal + 1,
                  u, unrm2, zpart, (i == 0 && k > 0) ? scal + 2 : nullptr, ud, vd};
      if (ps.ns == 16) launch_pass<512, 16, 1>(pa, L.parts, st);
      else if (ps.ns == 1) launch_pass<512, 1, 16>(pa, L.parts, st);
      else if (ps.ns == 2) launch_pass<512, 2, 8>(pa, L.parts, st);
      else if (ps.ns == 4) launch_pass<512, 4, 4>(pa, L.parts, st);
      else if (ps.ns == 6) launch_pass<512, 6, 2>(pa, L.parts, st);
      else launch_pass<512, 8, 1>(pa, L.parts, st);
      ReduceArgs ra{zpart, L.parts, (int)n, z, normpart, scal, scal + 1, counter};
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
