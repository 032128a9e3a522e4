// The forms of the scaled rank-one sketching loop (paper Sec. 3.3, Eq. 9-11; Algorithm 1, inner loop)
// that use a bfloat16 weight as it is handed over: the running matrix
//     A_k = W diag(s) - sum_{j<k} sigma_j U_j V_j^T      (stored factors)
// is never formed, its products are taken from W and the stored ranks enter as corrections.
// "stream" reads row blocks of W from memory in every application; "resident" keeps W on the chip.
#include "r1svd_device.h"

#include <cstdlib>
#include <cstring>

namespace ptq {
namespace {

using namespace r1svd_detail;

// ---- the loop on a bfloat16 weight that is never rewritten ------------------------------------
// The running matrix of rank k is  A_k = W diag(s) - sum_{j<k} sigma_j U_j V_j^T  with the STORED
// factors.  Instead of keeping A_k in memory (float32, rewritten at every rank) the products are
// taken from the weight as it was handed over:
//     u = A_k v   = W (s o v)     - sum_j sigma_j U_j (V_j . v)
//     z = A_k^T u = s o (W^T u)   - sum_j sigma_j V_j (U_j . u)
// so that an application streams 2 bytes per entry instead of 4, nothing is ever written back,
// and the first pass that builds W diag(s) disappears.  The corrections are small: a workgroup
// owns a contiguous range of rows and every 256th block of 16 columns, keeps the decoded entries
// of all U_j for its rows and of all V_j for its columns in LDS, and
//   * the k numbers V_j . v are summed over the columns as they are produced (each workgroup adds
//     its columns' share when it finishes them; the partial sums cross the grid barrier that ends
//     the application anyway),
//   * the k numbers U_j . u are summed over a workgroup's rows while it streams them and cross
//     the barrier that precedes the summation of the partial z vectors.
// Every sum has a fixed order.  The float32 scale fl(s) is used on both sides, so the matrix the
// loop sees is W diag(fl(s)): a relative change of 2^-24 per column, the size of the rounding
// the float32 copy of A makes in the other forms.

struct StreamArgs {
  const uint16_t* W; int64_t ldw; int m, n;
  const float* sf;          // n: the activation scale rounded to float32
  const float* S; int64_t lds; int r, it;
  uint8_t* U; uint8_t* V; uint16_t* sigma16;
  float* zpart; double* z; double* u; double* unrm2; double* normpart;
  double* cpart;            // [kMaxStreamRank][kComputeUnits]: shares of V_j . v
  double* dpart;            // [kMaxStreamRank][kComputeUnits]: shares of U_j . u
  float* zapp; int64_t zstride;
  int* expo; unsigned* bar; int* abort; unsigned spin_limit;
  int rows_own, cols_own;   // row lengths of the two LDS tables
};

__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xffff0000u); }

// R rows of W, 8 adjacent columns per thread in each of NS sweeps of 8 T columns, two bfloat16 per
// register.
template <int T, int NS, int R>
struct PackedRowBlock {
  unsigned w[NS][R][4];

  // rows row0 .. row0+R-1 below row_end (zeros beyond, and beyond column n)
  __device__ __forceinline__ void load(const uint16_t* W, int64_t ldw, int n, int row0, int row_end) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 8 * ((int)threadIdx.x + T * s);
#pragma unroll
      for (int i = 0; i < R; ++i) {
        uint4 q = make_uint4(0u, 0u, 0u, 0u);
        if (col < n && row0 + i < row_end) q = *reinterpret_cast<const uint4*>(W + (int64_t)(row0 + i) * ldw + col);
        w[s][i][0] = q.x; w[s][i][1] = q.y; w[s][i][2] = q.z; w[s][i][3] = q.w;
      }
    }
  }

  // us[i] = this thread's share of (row i) . (s o v),  v = vin * rs
  __device__ __forceinline__ void times_vector(const float* vin, const float* sf, float rs, int n, float (&us)[R]) const {
#pragma unroll
    for (int i = 0; i < R; ++i) us[i] = 0.f;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int col = 8 * ((int)threadIdx.x + T * s);
      float sv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      if (col < n) {
        const float4 v0 = *reinterpret_cast<const float4*>(vin + col), v1 = *reinterpret_cast<const float4*>(vin + col + 4);
        const float4 s0 = *reinterpret_cast<const float4*>(sf + col), s1 = *reinterpret_cast<const float4*>(sf + col + 4);
        sv[0] = v0.x * rs * s0.x; sv[1] = v0.y * rs * s0.y; sv[2] = v0.z * rs * s0.z; sv[3] = v0.w * rs * s0.w;
        sv[4] = v1.x * rs * s1.x; sv[5] = v1.y * rs * s1.y; sv[6] = v1.z * rs * s1.z; sv[7] = v1.w * rs * s1.w;
      }
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          us[i] = fmaf(bf16_hi(w[s][i][c]), sv[2 * c + 1], fmaf(bf16_lo(w[s][i][c]), sv[2 * c], us[i]));
    }
  }

  // zacc += (block)^T uf
  __device__ __forceinline__ void transposed_times(const float (&uf)[R], double (&zacc)[NS][8]) {
    // the packed words are unpacked again here: kept from times_vector, the unpacked floats would
    // take twice the registers of the block for the whole reduction in between
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) asm volatile("" : "+v"(w[s][i][c]));
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      float zt[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          zt[2 * c] = fmaf(bf16_lo(w[s][i][c]), uf[i], zt[2 * c]);
          zt[2 * c + 1] = fmaf(bf16_hi(w[s][i][c]), uf[i], zt[2 * c + 1]);
        }
#pragma unroll
      for (int c = 0; c < 8; ++c) zacc[s][c] += (double)zt[c];
    }
  }
};

// sum over the workgroups of one row of a [kMaxStreamRank][kComputeUnits] table, by one wave
__device__ __forceinline__ double share_sum(const double* row, int G) {
  double x[kComputeUnits / kWave];
#pragma unroll
  for (int q = 0; q < kComputeUnits / kWave; ++q) {
    const int p = (int)(threadIdx.x & 63) + q * kWave;
    const double v = load_dev(row + (p < G ? p : G - 1));   // issued whatever p: loads under a condition wait for each other
    x[q] = p < G ? v : 0.0;
  }
  double t = 0.0;
#pragma unroll
  for (int q = 0; q < kComputeUnits / kWave; ++q) t += x[q];
  return wave_sum(t);
}

template <int NS, int R>
__global__ __launch_bounds__(kChainThreads) void stream_chain_kernel(StreamArgs a) {
  constexpr int T = kChainThreads;
  constexpr int kWaves = T / kWave;
  constexpr int kGroups = T / kReduceCols;
  constexpr int KR = kMaxStreamRank;
  extern __shared__ float own[];          // decoded U_j for the own rows, then V_j for the own columns
  __shared__ double red[kWaves * R];
  __shared__ double ush[R];
  __shared__ double sred[kGroups][kReduceCols];
  __shared__ double fin[kWaves];
  __shared__ double sc[KR], sd[KR], sig[KR];
  __shared__ double cacc[KR][kReduceCols];
  __shared__ float stage[kWaves * 512];   // per wave: 8 rows x 64 lanes on their way to the row sums
  float* Uown = own;
  float* Vown = own + (size_t)KR * a.rows_own;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, b = blockIdx.x, G = gridDim.x;
  const int m = a.m, n = a.n;
  const int r0 = (int)((int64_t)b * m / G), r1 = (int)((int64_t)(b + 1) * m / G);
  const int ncb = (n + kReduceCols - 1) / kReduceCols;
  unsigned phase = 0;
  int app = 0;

  for (int k = 0; k < a.r; ++k) {
    for (int i = 0; i <= a.it; ++i, ++app) {
      double zacc[NS][8];
#pragma unroll
      for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int c = 0; c < 8; ++c) zacc[s][c] = 0.0;
      double unrm2 = 0.0, dacc = 0.0;
      float rs = 1.f;
      if (i > 0) {
        int e = __hip_atomic_load(a.expo + app - 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        e = e == INT_MIN ? 0 : (e > 126 ? 126 : (e < -126 ? -126 : e));
        rs = scalbnf(1.f, -e);
      }
      // sigma_j (V_j . v) for the stored ranks, v being the scaled input of this application
      for (int j = wave; j < k; j += kWaves) {
        const double t = share_sum(a.cpart + (size_t)j * kComputeUnits, G);
        if (lane == 0) sc[j] = sig[j] * t * (double)rs;
      }
      __syncthreads();
      // ordinary loads of v are safe: each application's z has an address of its own
      const float* v_in = i == 0 ? a.S + (int64_t)k * a.lds : a.zapp + (int64_t)(app - 1) * a.zstride;
      for (int row0 = r0; row0 < r1; row0 += R) {
        const float* vin = v_in;
        const float* sf = a.sf;
        asm volatile("" : "+s"(vin), "+s"(sf));
        PackedRowBlock<T, NS, R> blk;
        blk.load(a.W, a.ldw, n, row0, r1);
        float us[R];
        blk.times_vector(vin, sf, rs, n, us);
        wave_row_sums_into<R>(us, red, stage + wave * 512);
        __syncthreads();
        if (tid < R) {
          double t = 0.0;
          if (row0 + tid < r1) {
#pragma unroll
            for (int wv = 0; wv < kWaves; ++wv) t += red[wv * R + tid];
            const float* uo = Uown + (row0 - r0 + tid);
            for (int j = 0; j < k; ++j) t -= sc[j] * (double)uo[(size_t)j * a.rows_own];
            a.u[row0 + tid] = t;
          }
          ush[tid] = t;
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
          for (int q = 0; q < R; ++q) unrm2 = fma(ush[q], ush[q], unrm2);
        }
        if (tid < k) {
          const float* uo = Uown + (size_t)tid * a.rows_own + (row0 - r0);
          const int cnt = r1 - row0 < R ? r1 - row0 : R;
          for (int q = 0; q < cnt; ++q) dacc = fma((double)uo[q], ush[q], dacc);
        }
        float uf[R];
#pragma unroll
        for (int q = 0; q < R; ++q) uf[q] = (float)ush[q];
        blk.transposed_times(uf, zacc);
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int col = 8 * (tid + T * s);
        if (col < n) {
          float* o = a.zpart + ((int64_t)(col / kReduceCols) * G + b) * kReduceCols + col % kReduceCols;
          store_dev4(o, (float)zacc[s][0], (float)zacc[s][1], (float)zacc[s][2], (float)zacc[s][3]);
          store_dev4(o + 4, (float)zacc[s][4], (float)zacc[s][5], (float)zacc[s][6], (float)zacc[s][7]);
        }
      }
      if (tid == 0) store_dev(a.unrm2 + b, unrm2);
      if (tid < k) store_dev(a.dpart + (size_t)tid * kComputeUnits + b, dacc);
      grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);

      // this workgroup's column blocks of z = s o (sum of the partial vectors) - correction
      const bool last_app = i == a.it;
      for (int j = wave; j < k; j += kWaves) {
        const double t = share_sum(a.dpart + (size_t)j * kComputeUnits, G);
        if (lane == 0) sd[j] = sig[j] * t;
      }
      if (tid < KR * kReduceCols) cacc[tid / kReduceCols][tid % kReduceCols] = 0.0;
      __syncthreads();
      int lc0 = 0;
      for (int cb = b; cb < ncb; cb += G, lc0 += kReduceCols) {
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
            zz *= (double)a.sf[col];
            const float* vo = Vown + lc0 + cl;
            for (int j = 0; j < k; ++j) zz -= sd[j] * (double)vo[(size_t)j * a.cols_own];
            const float zf = (float)zz;
            store_dev(a.zapp + (int64_t)app * a.zstride + col, zf);
            a.z[col] = zz;   // read back by this workgroup only
            if (!last_app)
              for (int j = 0; j < k; ++j) cacc[j][cl] = fma((double)vo[(size_t)j * a.cols_own], (double)zf, cacc[j][cl]);
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
      if (!last_app && tid < k) {
        double t = 0.0;
#pragma unroll
        for (int c = 0; c < kReduceCols; ++c) t += cacc[tid][c];
        store_dev(a.cpart + (size_t)tid * kComputeUnits + b, t);
      }
      grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);
    }

    // the stored triplet of rank k: every workgroup derives the same norms and sigma, encodes the
    // entries of U and V it produced itself and keeps their decoded values
    const double ny = sqrt(block_sum<T>(a.unrm2, G, fin));
    const double np = sqrt(block_sum<T>(a.normpart, ncb, fin));
    const bool dead = !(ny > 0.0) || !(np > 0.0);
    const uint16_t h = dead ? 0 : fp16_encode_pos(np / ny);
    if (tid == 0) sig[k] = fp16_decode_pos(h);
    if (b == 0 && tid == 0) a.sigma16[k] = h;
    for (int row = r0 + tid; row < r1; row += T) {
      const uint8_t c = dead ? 0 : e4m3_encode(a.u[row] / ny);
      a.U[(int64_t)k * m + row] = c;
      Uown[(size_t)k * a.rows_own + row - r0] = (float)e4m3_decode(c);
    }
    if (tid < kReduceCols) {
      int lc0 = 0;
      for (int cb = b; cb < ncb; cb += G, lc0 += kReduceCols) {
        const int col = cb * kReduceCols + tid;
        uint8_t c = 0;
        if (col < n) {
          c = dead ? 0 : e4m3_encode(a.z[col] / np);
          a.V[(int64_t)k * n + col] = c;
        }
        Vown[(size_t)k * a.cols_own + lc0 + tid] = (float)e4m3_decode(c);
      }
    }
    __syncthreads();
    // shares of V_j . S_{k+1}, the first input of the next rank: 32 lanes per stored rank
    if (k + 1 < a.r) {
      const int j = tid / 32, part = tid % 32;
      const float* Sn = a.S + (int64_t)(k + 1) * a.lds;
      double t = 0.0;
      if (j <= k) {
        int lc0 = 0;
        for (int cb = b; cb < ncb; cb += G, lc0 += kReduceCols) {
          const int col = cb * kReduceCols + part;
          if (part < kReduceCols && col < n)
            t = fma((double)Vown[(size_t)j * a.cols_own + lc0 + part], (double)Sn[col], t);
        }
      }
#pragma unroll
      for (int o = 8; o >= 1; o >>= 1) t += __shfl_xor(t, o);
      if (part == 0 && j <= k) store_dev(a.cpart + (size_t)j * kComputeUnits + b, t);
    }
    grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);
  }

  if (b == 0 && __hip_atomic_load(a.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
    for (int k = tid; k < a.r; k += T) a.sigma16[k] = 0x7e00;
}

// R = W - (sum_k sigma_k U_k V_k^T) diag(s)^-1 from the stored factors (Algorithm 1; float64
// arithmetic, one rounding): what the resident and stream forms hand to the quantizer.  One workgroup per
// 4 rows x 1024 columns.
__global__ __launch_bounds__(256) void stream_residual_kernel(const uint16_t* __restrict__ W, int64_t ldw, int m,
                                                             int n, int r, const uint8_t* __restrict__ U,
                                                             const uint8_t* __restrict__ V,
                                                             const uint16_t* __restrict__ sigma16,
                                                             const double* __restrict__ s, float* __restrict__ Rout,
                                                             int64_t ldr) {
  __shared__ double su[4][kMaxStreamRank];
  __shared__ double lut[256];   // decoded e4m3 codes: a table read instead of the arithmetic, 64 times per thread
  lut[threadIdx.x] = e4m3_decode((uint8_t)threadIdx.x);
  const int nb = (n + 1023) / 1024;
  const int c = ((int)(blockIdx.x % nb) * 256 + threadIdx.x) * 4;
  const int row0 = (int)(blockIdx.x / nb) * 4;
  if (threadIdx.x < 4 * kMaxStreamRank) {
    const int i = threadIdx.x / kMaxStreamRank, k = threadIdx.x % kMaxStreamRank;
    su[i][k] = (k < r && row0 + i < m) ? fp16_decode_pos(sigma16[k]) * e4m3_decode(U[(int64_t)k * m + row0 + i]) : 0.0;
  }
  __syncthreads();
  if (c >= n) return;
  double low[4][4] = {};
  for (int k = 0; k < r; ++k) {
    const unsigned codes = *reinterpret_cast<const unsigned*>(V + (int64_t)k * n + c);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const double v = lut[(codes >> (8 * q)) & 0xffu];
#pragma unroll
      for (int i = 0; i < 4; ++i) low[i][q] = fma(su[i][k], v, low[i][q]);
    }
  }
  double sc4[4];   // 1 / s: one division per column, not per entry (the result is rounded to float32 anyway)
#pragma unroll
  for (int q = 0; q < 4; ++q) sc4[q] = 1.0 / s[c + q];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (row0 + i >= m) break;
    const uint2 wv = *reinterpret_cast<const uint2*>(W + (int64_t)(row0 + i) * ldw + c);
    const double w4[4] = {(double)bf16_lo(wv.x), (double)bf16_hi(wv.x), (double)bf16_lo(wv.y), (double)bf16_hi(wv.y)};
    float o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = (float)(w4[q] - low[i][q] * sc4[q]);
    *reinterpret_cast<float4*>(Rout + (int64_t)(row0 + i) * ldr + c) = make_float4(o[0], o[1], o[2], o[3]);
  }
}

__global__ __launch_bounds__(256) void narrow_scale_kernel(const double* __restrict__ s, int n, float* __restrict__ sf) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c < n) sf[c] = (float)s[c];
}

// ---- the loop on a bfloat16 weight that fits the registers and LDS of the chip -----------------
// The same products as the stream form, but the weight is read ONCE: the matrix is cut into
// P x Q tiles (P Q <= 256), workgroup (p, q) keeps its tile for the whole loop -- 8 waves, a
// band of rows per wave, the first RR rows of a band packed in registers (128 per thread), the
// others in LDS -- and an application is
//   A  partial u of the tile from v (the tile's columns)            -> upart
//   B  u of the tile's rows = sum over the Q tiles of the row group - corrections
//   C  partial z of the tile from u                                  -> zpart
//   D  z of the tile's columns = s o (sum over the P tiles of the column group) - corrections
// so what crosses the chip is P n + Q m numbers per application instead of 256 n, and nothing
// is streamed.  There is no barrier inside an application: everything exchanged is a tagged
// word (float32 partial sums; the float64 dot products as a high and a low float32), and two
// buffers alternate.  A tile writes the words of application i + 2 only after it has seen those
// of application i + 1 from everybody it exchanges with, and each of them published those after
// it had read application i; for the dot products, which everybody reads, the same follows
// through one more exchange (row group, then column group, reach every tile).  Only the norms
// of a rank's last vectors meet at a grid barrier, once per rank.
// Every tile of a row group derives the same u, every tile of a column group the same z (same
// loads, same order), so the small jobs are shared out: of the dot products with the stored
// ranks tile (p, q) takes rank j = q (mod Q) for its row group and j = p (mod P) for its column
// group; of the norms it takes the q-th part of its rows and the p-th part of its columns.
// The power of two that keeps the vectors in range travels with the partial u (the exponent of
// the largest entry of the tile's columns of v; a row group sees all columns) and is applied
// to u, A being linear.  7B-sized MLP projections (90 MB) just fit: 352 KB per compute unit.
// Of a larger weight the rows of a band that fit neither registers nor LDS are re-read from
// memory, eight at a time, in step A and again in step C.
struct ResidentArgs {
  const uint16_t* W; int64_t ldw; int m, n;
  const float* sf; const float* S; int64_t lds; int r, it;
  uint8_t* U; uint8_t* V; uint16_t* sigma16;
  unsigned long long* upart;   // tagged [2][workgroup][kResidentRows]: partial u, then the exponent of the tile's v
  unsigned long long* zpart;   // tagged [2][workgroup][kResidentCols]: partial z
  unsigned long long* cpart;   // tagged [2][kMaxStreamRank][kComputeUnits][2]: (V_j . v) per column group
  unsigned long long* dpart;   // tagged [2][kMaxStreamRank][kComputeUnits][2]: (U_j . u) per row group
  double* unrm2; double* normpart;   // per workgroup
  unsigned* bar; int* abort; unsigned spin_limit;
  int P, Q, RW, RL;         // row groups, column groups, rows per wave, of which in LDS
};

// LDS of the resident form by tile shape; `shared` (8 x 512 floats) holds, at different times, the
// per-wave staging of step A's row sums, the per-wave column sums of step C, and the sums of the
// partial z and the float32 copy of z of step D.
struct ResidentLds {
  size_t tile, ush, ustage, shared, small, svsh, uf, lut, ucode, vcode, total;
};
__host__ __device__ inline ResidentLds resident_lds(int nsw, int rr, int rw, int rl) {
  const int tc = nsw * 512, tr = 8 * rw;
  const int chunks = rr / 8 + (rw > rr ? (rw - rr + 7) / 8 : 0);
  ResidentLds L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t at = off; off += (bytes + 15) & ~size_t{15}; return at; };
  L.tile = take((size_t)8 * rl * tc * 2);
  L.ush = take((size_t)tr * 8);
  L.ustage = take((size_t)chunks * 64 * 8);
  L.shared = take((size_t)8 * 512 * 4);
  L.small = take(64 * 8 + 16 * 4);
  L.svsh = take((size_t)tc * 4);
  L.uf = take((size_t)(tr + rr) * 4);
  L.lut = take(256 * 4);
  L.ucode = take((size_t)kMaxStreamRank * tr);
  L.vcode = take((size_t)kMaxStreamRank * tc);
  L.total = off;
  return L;
}

// A float64 as two tagged words: the nearest float32 and the float32 nearest to what is left.
__device__ __forceinline__ void store_tagged_pair(unsigned long long* p, double v, unsigned tag) {
  const float hi = (float)v;
  const float lo = (float)(v - (double)hi);
  store_tagged(p, __float_as_uint(hi), tag);
  store_tagged(p + 1, __float_as_uint(lo), tag);
}

// Sum over the first `count` slots of row j = thread / 32 of a tagged [kMaxStreamRank]
// [kComputeUnits][2] table, for the rows j < k; waits for the tag.  out[j] = sig[j] * sum.
__device__ __forceinline__ void tagged_share_sums(const unsigned long long* table, int count, int k, unsigned tag,
                                                  const double* sig, double* out, int* abort, unsigned spin_limit) {
  if (k == 0) return;
  const int j = threadIdx.x / 32, part = threadIdx.x % 32;
  const unsigned long long* row = table + (size_t)j * kComputeUnits * 2;
  double t = 0.0;
  unsigned spins = 0;
  for (int o0 = 0; o0 < count; o0 += 32) {
    const int o = o0 + part;
    const bool want = j < k && o < count;
    const unsigned long long* w2 = row + (size_t)(o < count ? o : count - 1) * 2;
    unsigned long long hi, lo;
    bool ready;
    do {
      hi = load_tagged(w2);
      lo = load_tagged(w2 + 1);
      ready = !want || ((unsigned)(hi >> 32) == tag && (unsigned)(lo >> 32) == tag);
    } while (!ready && keep_waiting(spins, abort, spin_limit));
    t += want ? (double)__uint_as_float((unsigned)hi) + (double)__uint_as_float((unsigned)lo) : 0.0;
  }
  t = sum32(t);
  if (part == 0 && j < k) out[j] = sig[j] * t;
}

// (decoded codes of rank j) . vec over `len` entries, for the ranks j < k that fall to this
// workgroup (j = owner modulo owners), left in out[j][slot] as a tagged pair.  The whole
// workgroup works on one rank at a time (an entry per thread, then a sum over the workgroup in
// a fixed order); the codes of an entry's 16 ranks are adjacent.  Contains workgroup barriers;
// `scratch`: 8 doubles.
template <typename VT>
__device__ __forceinline__ void dot_shares(const uint8_t* codes, const float* lut, const VT* vec, int len, int k,
                                           int owners, int owner, int slot, unsigned long long* out, unsigned tag,
                                           double* scratch) {
  const int tid = threadIdx.x;
  for (int j = owner; j < k; j += owners) {
    double t = 0.0;
    for (int x = tid; x < len; x += kChainThreads)
      t = fma((double)lut[codes[(size_t)x * kMaxStreamRank + j]], (double)vec[x], t);
    t = sum32(t);
    t += __shfl_xor(t, 32);
    if ((tid & 63) == 0) scratch[tid >> 6] = t;
    __syncthreads();
    if (tid == 0) {
      double total = 0.0;
#pragma unroll
      for (int wv = 0; wv < kChainThreads / kWave; ++wv) total += scratch[wv];
      store_tagged_pair(out + ((size_t)j * kComputeUnits + slot) * 2, total, tag);
    }
    __syncthreads();
  }
}

// sum_j coef[j] * (decoded code j of the 16 adjacent codes at `codes`), j < k
__device__ __forceinline__ double stored_ranks_dot(const uint8_t* codes, const float* lut, const double* coef, int k) {
  const uint4 cw = *reinterpret_cast<const uint4*>(codes);
  const unsigned wd[4] = {cw.x, cw.y, cw.z, cw.w};
  double t = 0.0;
#pragma unroll
  for (int j = 0; j < kMaxStreamRank; ++j) {
    const float v = lut[(wd[j >> 2] >> (8 * (j & 3))) & 0xffu];
    t += j < k ? coef[j] * (double)v : 0.0;
  }
  return t;
}

template <int NSW, int RR>
__global__ __launch_bounds__(kChainThreads) void resident_chain_kernel(ResidentArgs a) {
  constexpr int T = kChainThreads, KR = kMaxStreamRank, TC = NSW * 512;
  static_assert(T == 512 && KR * 32 == T, "32 lanes per stored rank");
  extern __shared__ __align__(16) unsigned char lds_raw[];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, b = blockIdx.x, G = gridDim.x;
  const int p = b / a.Q, q = b % a.Q, P = a.P, Q = a.Q;
  const int m = a.m, n = a.n, RW = a.RW, TR = 8 * RW, RL = a.RL;
  const int RG = RW - RR - RL > 0 ? RW - RR - RL : 0;   // rows of a band that fit neither: read from memory in A and in C
  const ResidentLds L = resident_lds(NSW, RR, RW, RL);
  uint4* tile = reinterpret_cast<uint4*>(lds_raw + L.tile);
  double* ush = reinterpret_cast<double*>(lds_raw + L.ush);
  double* ustage = reinterpret_cast<double*>(lds_raw + L.ustage);
  float* stage = reinterpret_cast<float*>(lds_raw + L.shared) + w * 512;
  float* zred = reinterpret_cast<float*>(lds_raw + L.shared);
  float* vsh = reinterpret_cast<float*>(lds_raw + L.shared);
  double* sc = reinterpret_cast<double*>(lds_raw + L.small);
  double* sd = sc + 16; double* sig = sc + 32; double* fin = sc + 48;
  int* esh = reinterpret_cast<int*>(sc + 64);
  float* svsh = reinterpret_cast<float*>(lds_raw + L.svsh);
  float* uf = reinterpret_cast<float*>(lds_raw + L.uf);
  float* lut = reinterpret_cast<float*>(lds_raw + L.lut);
  uint8_t* ucode = lds_raw + L.ucode;
  uint8_t* vcode = lds_raw + L.vcode;

  // ---- the tile, once
  unsigned wreg[RR][NSW][4];
#pragma unroll
  for (int rr = 0; rr < RR; ++rr)
#pragma unroll
    for (int s = 0; s < NSW; ++s) {
      const int row = p * TR + w * RW + rr, col = q * TC + s * 512 + lane * 8;
      uint4 x = make_uint4(0u, 0u, 0u, 0u);
      if (rr < RW && row < m && col < n) x = *reinterpret_cast<const uint4*>(a.W + (int64_t)row * a.ldw + col);
      wreg[rr][s][0] = x.x; wreg[rr][s][1] = x.y; wreg[rr][s][2] = x.z; wreg[rr][s][3] = x.w;
    }
  for (int rl = 0; rl < RL; ++rl)
#pragma unroll
    for (int s = 0; s < NSW; ++s) {
      const int row = p * TR + w * RW + RR + rl, col = q * TC + s * 512 + lane * 8;
      uint4 x = make_uint4(0u, 0u, 0u, 0u);
      if (row < m && col < n) x = *reinterpret_cast<const uint4*>(a.W + (int64_t)row * a.ldw + col);
      tile[(size_t)(w * RL + rl) * (TC / 8) + s * 64 + lane] = x;
    }
  // kStreamRows rows of the wave's band from memory, from row r0 on; all loads are issued before the
  // first is used (rows past the band or the matrix are fetched from a valid row and zeroed)
  constexpr int kStreamRows = 8 / NSW;
  auto streamed_rows = [&](uint4 (&g4)[kStreamRows][NSW], int r0) {
#pragma unroll
    for (int x = 0; x < kStreamRows; ++x)
#pragma unroll
      for (int s = 0; s < NSW; ++s) {
        const int row = p * TR + w * RW + r0 + x, col = q * TC + s * 512 + lane * 8;
        const bool live = r0 + x < RW && row < m && col < n;
        const uint4 v = *reinterpret_cast<const uint4*>(a.W + (int64_t)(row < m ? row : m - 1) * a.ldw + (col < n ? col : 0));
        g4[x][s] = live ? v : make_uint4(0u, 0u, 0u, 0u);
      }
  };
  if (tid < 256) lut[tid] = (float)e4m3_decode((uint8_t)tid);
  for (int x = tid; x < TR + RR; x += T) uf[x] = 0.f;
  float sfc[NSW];
#pragma unroll
  for (int s = 0; s < NSW; ++s) {
    const int gcol = q * TC + s * 512 + tid;
    sfc[s] = gcol < n ? a.sf[gcol] : 0.f;
    svsh[s * 512 + tid] = gcol < n ? a.S[gcol] * sfc[s] : 0.f;
  }
  __syncthreads();

  const int row_lo = (int)((int64_t)q * TR / Q), row_hi = (int)((int64_t)(q + 1) * TR / Q);
  const int col_lo = (int)((int64_t)p * TC / P), col_hi = (int)((int64_t)(p + 1) * TC / P);
  unsigned phase = 0;
  unsigned app = 0;       // applications so far: the tag of what this one exchanges
  int ecol = INT_MIN;     // exponent of the largest entry of this tile's columns of v (INT_MIN: do not scale)

  for (int k = 0; k < a.r; ++k) {
    double zcur[NSW];
    for (int i = 0; i <= a.it; ++i) {
      const bool last_app = i == a.it;
      ++app;
      unsigned long long* const up = a.upart + ((size_t)(app & 1u) * G + b) * kResidentRows;
      unsigned long long* const zp = a.zpart + ((size_t)(app & 1u) * G + b) * kResidentCols;
      const unsigned long long* const cin = a.cpart + (size_t)(app & 1u) * kShareWords;
      unsigned long long* const dio = a.dpart + (size_t)(app & 1u) * kShareWords;
      unsigned long long* const cout = a.cpart + (size_t)((app + 1) & 1u) * kShareWords;
      // ---- A: partial u of the tile
      {
        float sv[NSW][8];
#pragma unroll
        for (int s = 0; s < NSW; ++s) {
          const float4 x = *reinterpret_cast<const float4*>(svsh + s * 512 + lane * 8);
          const float4 y = *reinterpret_cast<const float4*>(svsh + s * 512 + lane * 8 + 4);
          sv[s][0] = x.x; sv[s][1] = x.y; sv[s][2] = x.z; sv[s][3] = x.w;
          sv[s][4] = y.x; sv[s][5] = y.y; sv[s][6] = y.z; sv[s][7] = y.w;
        }
#pragma unroll
        for (int c8 = 0; c8 < RR / 8; ++c8) {
          if (c8 * 8 < RW) {
            float us[8];
#pragma unroll
            for (int x = 0; x < 8; ++x) {
              us[x] = 0.f;
#pragma unroll
              for (int s = 0; s < NSW; ++s)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                  us[x] = fmaf(bf16_hi(wreg[c8 * 8 + x][s][c]), sv[s][2 * c + 1],
                               fmaf(bf16_lo(wreg[c8 * 8 + x][s][c]), sv[s][2 * c], us[x]));
            }
            const double t = wave_row_sums_staged(us, stage);
            if ((lane & 7) == 0) ustage[c8 * 64 + w * 8 + (lane >> 3)] = t;
          }
        }
        for (int c8 = RR / 8; c8 * 8 < RR + RL; ++c8) {
          float us[8];
#pragma unroll
          for (int x = 0; x < 8; ++x) {
            us[x] = 0.f;
            const int rl = c8 * 8 - RR + x;
            if (rl < RL) {
#pragma unroll
              for (int s = 0; s < NSW; ++s) {
                const uint4 t4 = tile[(size_t)(w * RL + rl) * (TC / 8) + s * 64 + lane];
                const unsigned wd[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                  us[x] = fmaf(bf16_hi(wd[c]), sv[s][2 * c + 1], fmaf(bf16_lo(wd[c]), sv[s][2 * c], us[x]));
              }
            }
          }
          const double t = wave_row_sums_staged(us, stage);
          if ((lane & 7) == 0) ustage[c8 * 64 + w * 8 + (lane >> 3)] = t;
        }
        // rows beyond registers and LDS (RR + RL is then a multiple of 8): eight at a time from memory
        for (int c8 = (RR + RL) / 8; c8 * 8 < RW && RG > 0; ++c8) {
          float us[8];
#pragma unroll
          for (int x0 = 0; x0 < 8; x0 += kStreamRows) {
            uint4 g4[kStreamRows][NSW];
            streamed_rows(g4, c8 * 8 + x0);
#pragma unroll
            for (int x = 0; x < kStreamRows; ++x) {
              float t = 0.f;
#pragma unroll
              for (int s = 0; s < NSW; ++s) {
                const unsigned wd[4] = {g4[x][s].x, g4[x][s].y, g4[x][s].z, g4[x][s].w};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                  t = fmaf(bf16_hi(wd[c]), sv[s][2 * c + 1], fmaf(bf16_lo(wd[c]), sv[s][2 * c], t));
              }
              us[x0 + x] = t;
            }
          }
          const double t = wave_row_sums_staged(us, stage);
          if ((lane & 7) == 0) ustage[c8 * 64 + w * 8 + (lane >> 3)] = t;
        }
      }
      __syncthreads();
      if (tid < TR) {
        const int wv = tid / RW, x = tid - wv * RW;
        store_tagged(up + tid, __float_as_uint((float)ustage[(x >> 3) * 64 + wv * 8 + (x & 7)]), app);
      } else if (tid == TR) {
        store_tagged(up + TR, (unsigned)ecol, app);
      }

      // ---- B: u of the row group.  Thread t < TR adds up row t's partial sums, thread TR takes the
      // largest of the exponents; all loads of a round are issued before the first is looked at.
      double usum = 0.0;
      {
        constexpr int kBatch = 12;
        const unsigned long long* src = a.upart + ((size_t)(app & 1u) * G + (size_t)p * Q) * kResidentRows + (tid < TR ? tid : TR);
        int e_in = INT_MIN;
        unsigned spins = 0;
        for (int q0 = 0; q0 < Q; q0 += kBatch) {
          const int cnt = Q - q0 < kBatch ? Q - q0 : kBatch;
          unsigned long long x[kBatch];
          bool ready;
          do {
            ready = true;
#pragma unroll
            for (int j = 0; j < kBatch; ++j) {
              x[j] = load_tagged(src + (size_t)(q0 + (j < cnt ? j : cnt - 1)) * kResidentRows);
              ready = ready && (unsigned)(x[j] >> 32) == app;
            }
          } while (!ready && keep_waiting(spins, a.abort, a.spin_limit));
#pragma unroll
          for (int j = 0; j < kBatch; ++j) {
            usum += j < cnt ? (double)__uint_as_float((unsigned)x[j]) : 0.0;
            e_in = max(e_in, j < cnt ? (int)(unsigned)x[j] : INT_MIN);
          }
        }
        if (tid == TR) esh[0] = e_in;
        tagged_share_sums(cin, Q, k, app, sig, sc, a.abort, a.spin_limit);
      }
      __syncthreads();
      const double rs = unscale(esh[0]);
      if (tid < TR) {
        const double t = (usum - stored_ranks_dot(ucode + (size_t)tid * KR, lut, sc, k)) * rs;
        ush[tid] = t;
        uf[tid] = (float)t;
      }
      __syncthreads();
      dot_shares(ucode, lut, ush, TR, k, Q, q, p, dio, app, fin);
      if (last_app) {
        const double x = (tid >= row_lo && tid < row_hi) ? ush[tid] * ush[tid] : 0.0;
        const double t = wave_sum(x);
        if (lane == 0) fin[w] = t;
        __syncthreads();
        if (tid == 0) {
          double total = 0.0;
#pragma unroll
          for (int wv = 0; wv < T / kWave; ++wv) total += fin[wv];
          store_dev(a.unrm2 + b, total);
        }
      }

      // ---- C: partial z of the tile
      {
        float zt[NSW][8];
#pragma unroll
        for (int s = 0; s < NSW; ++s)
#pragma unroll
          for (int c = 0; c < 8; ++c) zt[s][c] = 0.f;
        // the packed words are unpacked again: unpacked floats kept from step A, or hoisted out of
        // the loop, would need twice the registers of the tile
#pragma unroll
        for (int rr = 0; rr < RR; ++rr)
#pragma unroll
          for (int s = 0; s < NSW; ++s)
#pragma unroll
            for (int c = 0; c < 4; ++c) asm volatile("" : "+v"(wreg[rr][s][c]));
#pragma unroll
        for (int rr = 0; rr < RR; ++rr) {
          const float ufv = uf[w * RW + rr];   // rows past the band hold zeros in wreg
#pragma unroll
          for (int s = 0; s < NSW; ++s)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              zt[s][2 * c] = fmaf(bf16_lo(wreg[rr][s][c]), ufv, zt[s][2 * c]);
              zt[s][2 * c + 1] = fmaf(bf16_hi(wreg[rr][s][c]), ufv, zt[s][2 * c + 1]);
            }
        }
        for (int rl = 0; rl < RL; ++rl) {
          const float ufv = uf[w * RW + RR + rl];
#pragma unroll
          for (int s = 0; s < NSW; ++s) {
            const uint4 t4 = tile[(size_t)(w * RL + rl) * (TC / 8) + s * 64 + lane];
            const unsigned wd[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              zt[s][2 * c] = fmaf(bf16_lo(wd[c]), ufv, zt[s][2 * c]);
              zt[s][2 * c + 1] = fmaf(bf16_hi(wd[c]), ufv, zt[s][2 * c + 1]);
            }
          }
        }
        for (int r0 = RR + RL; r0 < RW; r0 += kStreamRows) {
          uint4 g4[kStreamRows][NSW];
          streamed_rows(g4, r0);
#pragma unroll
          for (int x = 0; x < kStreamRows; ++x) {
            const float ufv = r0 + x < RW ? uf[w * RW + r0 + x] : 0.f;
#pragma unroll
            for (int s = 0; s < NSW; ++s) {
              const unsigned wd[4] = {g4[x][s].x, g4[x][s].y, g4[x][s].z, g4[x][s].w};
#pragma unroll
              for (int c = 0; c < 4; ++c) {
                zt[s][2 * c] = fmaf(bf16_lo(wd[c]), ufv, zt[s][2 * c]);
                zt[s][2 * c + 1] = fmaf(bf16_hi(wd[c]), ufv, zt[s][2 * c + 1]);
              }
            }
          }
        }
#pragma unroll
        for (int s = 0; s < NSW; ++s) {
          __syncthreads();   // the shared region: step A's sums were read before the barrier, sweep s - 1 just above
          *reinterpret_cast<float4*>(zred + w * 512 + lane * 8) = make_float4(zt[s][0], zt[s][1], zt[s][2], zt[s][3]);
          *reinterpret_cast<float4*>(zred + w * 512 + lane * 8 + 4) = make_float4(zt[s][4], zt[s][5], zt[s][6], zt[s][7]);
          __syncthreads();
          double t = 0.0;
#pragma unroll
          for (int wv = 0; wv < T / kWave; ++wv) t += (double)zred[wv * 512 + tid];
          store_tagged(zp + s * 512 + tid, __float_as_uint((float)t), app);
        }
      }

      // ---- D: z of the column group, the next input
      double zsum[NSW];
      {
        constexpr int kBatch = 16;
        unsigned spins = 0;
#pragma unroll
        for (int s = 0; s < NSW; ++s) {
          zsum[s] = 0.0;
          const unsigned long long* src = a.zpart + ((size_t)(app & 1u) * G + q) * kResidentCols + s * 512 + tid;
          for (int p0 = 0; p0 < P; p0 += kBatch) {
            const int cnt = P - p0 < kBatch ? P - p0 : kBatch;
            unsigned long long x[kBatch];
            bool ready;
            do {
              ready = true;
#pragma unroll
              for (int j = 0; j < kBatch; ++j) {
                x[j] = load_tagged(src + (size_t)(p0 + (j < cnt ? j : cnt - 1)) * Q * kResidentCols);
                ready = ready && (unsigned)(x[j] >> 32) == app;
              }
            } while (!ready && keep_waiting(spins, a.abort, a.spin_limit));
#pragma unroll
            for (int j = 0; j < kBatch; ++j) zsum[s] += j < cnt ? (double)__uint_as_float((unsigned)x[j]) : 0.0;
          }
        }
        tagged_share_sums(dio, P, k, app, sig, sd, a.abort, a.spin_limit);
      }
      __syncthreads();
      int e = INT_MIN;
      double q2 = 0.0;
#pragma unroll
      for (int s = 0; s < NSW; ++s) {
        const int cl = s * 512 + tid;
        double zz = zsum[s] * (double)sfc[s] - stored_ranks_dot(vcode + (size_t)cl * KR, lut, sd, k);
        if (q * TC + cl >= n) zz = 0.0;
        zcur[s] = zz;
        const float zf = (float)zz;
        vsh[cl] = zf;
        svsh[cl] = zf * sfc[s];
        if (zz != 0.0 && fabs(zz) < __builtin_inf()) e = max(e, ilogb(zz));
        if (cl >= col_lo && cl < col_hi) q2 = fma(zz, zz, q2);
      }
      __syncthreads();
      if (!last_app) {
        dot_shares(vcode, lut, vsh, TC, k, P, p, q, cout, app + 1, fin);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) e = max(e, __shfl_xor(e, o));
        if (lane == 0) esh[1 + w] = e;
        __syncthreads();
        ecol = INT_MIN;
#pragma unroll
        for (int wv = 0; wv < T / kWave; ++wv) ecol = max(ecol, esh[1 + wv]);
      } else {
        ecol = INT_MIN;   // the next rank starts from a sketch vector
        const double t = wave_sum(q2);
        if (lane == 0) fin[w] = t;
        __syncthreads();
        if (tid == 0) {
          double total = 0.0;
#pragma unroll
          for (int wv = 0; wv < T / kWave; ++wv) total += fin[wv];
          store_dev(a.normpart + b, total);
        }
      }
    }
    grid_barrier(a.bar, ++phase, a.abort, a.spin_limit);

    // ---- the stored triplet of rank k
    const double ny = sqrt(block_sum<T>(a.unrm2, G, fin));
    const double np = sqrt(block_sum<T>(a.normpart, G, fin));
    const bool dead = !(ny > 0.0) || !(np > 0.0);
    const uint16_t h = dead ? 0 : fp16_encode_pos(np / ny);
    if (tid == 0) sig[k] = fp16_decode_pos(h);
    if (b == 0 && tid == 0) a.sigma16[k] = h;
    if (tid < TR) {
      const int row = p * TR + tid;
      const uint8_t c = (dead || row >= m) ? 0 : e4m3_encode(ush[tid] / ny);
      ucode[(size_t)tid * KR + k] = c;
      if (q == 0 && row < m) a.U[(int64_t)k * m + row] = c;
    }
#pragma unroll
    for (int s = 0; s < NSW; ++s) {
      const int cl = s * 512 + tid, gcol = q * TC + cl;
      const uint8_t c = (dead || gcol >= n) ? 0 : e4m3_encode(zcur[s] / np);
      vcode[(size_t)cl * KR + k] = c;
      if (p == 0 && gcol < n) a.V[(int64_t)k * n + gcol] = c;
      if (k + 1 < a.r) {
        const float x = gcol < n ? a.S[(int64_t)(k + 1) * a.lds + gcol] : 0.f;
        vsh[cl] = x;
        svsh[cl] = x * sfc[s];
      }
    }
    __syncthreads();
    if (k + 1 < a.r)
      dot_shares(vcode, lut, vsh, TC, k + 1, P, p, q, a.cpart + (size_t)((app + 1) & 1u) * kShareWords, app + 1, fin);
    __syncthreads();   // vsh shares its memory with step A's sums
  }

  if (b == 0 && __hip_atomic_load(a.abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)
    for (int k = tid; k < a.r; k += T) a.sigma16[k] = 0x7e00;
}

// ---- host side -----------------------------------------------------------------------------------
// Shape of the stream form by number of columns: 8 * sweeps * rows bfloat16 of W per thread.
struct StreamShape { int ns, rows; };
inline StreamShape stream_shape(int64_t n) {
  if (n <= 4096) return {1, 16};
  if (n <= 8192) return {2, 8};
  if (n <= 12288) return {3, 4};
  return {4, 4};
}

template <int NS, int R>
bool launch_stream(StreamArgs& a, hipStream_t st) {
  const int64_t ncb = ceil_div((int64_t)a.n, kReduceCols);
  const int64_t want = ceil_div((int64_t)a.m, R) > ncb ? ceil_div((int64_t)a.m, R) : ncb;
  const int groups = (int)(want < kComputeUnits ? want : kComputeUnits);
  a.rows_own = (int)ceil_div((int64_t)a.m, groups);
  a.cols_own = (int)ceil_div(ncb, groups) * kReduceCols;
  const size_t lds = (size_t)kMaxStreamRank * (a.rows_own + a.cols_own) * sizeof(float);
  constexpr size_t kMaxLds = 96 * 1024;
  if (lds > kMaxLds || !lds_opt_in<stream_chain_kernel<NS, R>>((int)kMaxLds)) return false;
  int dev = 0, coop = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, stream_chain_kernel<NS, R>, kChainThreads, lds) != hipSuccess)
    return false;
  if ((int64_t)per_cu * cus < groups) return false;
  void* params[] = {&a};
  if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(stream_chain_kernel<NS, R>), dim3((unsigned)groups),
                                 dim3(kChainThreads), params, (unsigned)lds, st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

// Tile shape of the resident form: column sweeps per tile (512 columns each), rows per wave, groups.
constexpr size_t kResidentMaxLds = 160 * 1024;
struct ResidentPlan { int nsw, rr, rw, rl, P, Q; size_t lds; bool ok; };
inline ResidentPlan resident_plan(int64_t m, int64_t n) {
  ResidentPlan best{};
  int64_t best_cost = 0;
  for (int nsw = 1; nsw <= 2; ++nsw) {
    const int rr = 32 / nsw;
    const int64_t Q = ceil_div(n, (int64_t)512 * nsw);
    if (Q > kComputeUnits) continue;
    int64_t P = kComputeUnits / Q;
    const int64_t rw = ceil_div(m, 8 * P);
    P = ceil_div(m, 8 * rw);
    if (8 * rw >= kResidentRows) continue;   // a row per thread, and the word after the rows
    // rows of a band: rr in registers, as many of the others as LDS holds, the rest re-read from
    // memory twice per application (in whole groups of 8, so LDS rows are then a multiple of 8)
    const size_t fixed = resident_lds(nsw, rr, (int)rw, 0).total;
    if (fixed > kResidentMaxLds) continue;
    const int64_t row_bytes = (int64_t)8 * 512 * nsw * 2;
    int64_t rl = rw > rr ? rw - rr : 0;
    const int64_t room = (int64_t)(kResidentMaxLds - fixed) / row_bytes;
    if (rl > room) rl = room / 8 * 8;
    const int64_t rg = rw - rr - rl > 0 ? rw - rr - rl : 0;
    if (rg * 4 > rw * 3) continue;           // mostly streamed: the stream form is the better fit
    const int64_t cost = (rw + 2 * rg) * nsw;   // a streamed row costs about three resident ones
    if (!best.ok || cost < best_cost) {
      best = {nsw, rr, (int)rw, (int)rl, (int)P, (int)Q, resident_lds(nsw, rr, (int)rw, (int)rl).total, true};
      best_cost = cost;
    }
  }
  return best;
}

template <int NSW, int RR>
bool launch_resident(ResidentArgs& a, const ResidentPlan& plan, hipStream_t st) {
  if (!lds_opt_in<resident_chain_kernel<NSW, RR>>((int)kResidentMaxLds)) return false;
  int dev = 0, coop = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev) != hipSuccess || !coop) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, resident_chain_kernel<NSW, RR>, kChainThreads, plan.lds) !=
      hipSuccess)
    return false;
  const int groups = plan.P * plan.Q;
  if ((int64_t)per_cu * cus < groups) return false;
  void* params[] = {&a};
  if (hipLaunchCooperativeKernel(reinterpret_cast<const void*>(resident_chain_kernel<NSW, RR>), dim3((unsigned)groups),
                                 dim3(kChainThreads), params, (unsigned)plan.lds, st) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return true;
}

}  // namespace

bool r1svd_bf16_launch(const R1svdBf16Call& c, hipStream_t st) {
  const int64_t m = c.m, n = c.n;
  const int apps = c.r * (c.it + 1);
  const int init = apps > kBarrierWords ? apps : kBarrierWords;
  narrow_scale_kernel<<<(unsigned)ceil_div(n, 256), 256, 0, st>>>(c.s, (int)n, c.sf);
  chain_init_kernel<<<(unsigned)ceil_div(init, 256), 256, 0, st>>>(c.expo, apps, c.bar, c.abort_flag);
  bool launched = false;
  const ResidentPlan plan = resident_plan(m, n);
  if (plan.ok && !c.stream_only) {
    char* rw = c.resident_ws;
    // tags of an earlier call must not be mistaken for this one's: the tagged words start at zero
    const int words = (int)(kResidentWorkspaceBytes / sizeof(unsigned));
    tile_init_kernel<<<(unsigned)ceil_div(words, 256), 256, 0, st>>>(reinterpret_cast<unsigned*>(rw), words, c.abort_flag);
    ResidentArgs ra{c.W, c.ldw, (int)m, (int)n, c.sf, c.S, c.lds, c.r, c.it, c.U, c.V, c.sigma16,
                    reinterpret_cast<unsigned long long*>(rw),
                    reinterpret_cast<unsigned long long*>(rw + kResidentUpartBytes),
                    reinterpret_cast<unsigned long long*>(rw + kResidentUpartBytes + kResidentZpartBytes),
                    reinterpret_cast<unsigned long long*>(rw + kResidentUpartBytes + kResidentZpartBytes + kResidentShareBytes),
                    c.unrm2, c.normpart, c.bar, c.abort_flag, c.spin_limit, plan.P, plan.Q, plan.rw, plan.rl};
    launched = plan.nsw == 1 ? launch_resident<1, 32>(ra, plan, st) : launch_resident<2, 16>(ra, plan, st);
  }
  if (!launched) {
    StreamArgs sa{c.W, c.ldw, (int)m, (int)n, c.sf, c.S, c.lds, c.r, c.it, c.U, c.V, c.sigma16,
                  c.zpart, c.z, c.u, c.unrm2, c.normpart, c.shares, c.shares + (size_t)kMaxStreamRank * kComputeUnits,
                  c.zapp, c.zstride, c.expo, c.bar, c.abort_flag, c.spin_limit, 0, 0};
    switch (stream_shape(n).ns) {
      case 1: launched = launch_stream<1, 16>(sa, st); break;
      case 2: launched = launch_stream<2, 8>(sa, st); break;
      case 3: launched = launch_stream<3, 4>(sa, st); break;
      default: launched = launch_stream<4, 4>(sa, st); break;
    }
  }
  if (!launched) return false;
  // the residual from W and the stored codes
  const unsigned gr = (unsigned)(ceil_div(n, 1024) * ceil_div(m, 4));
  stream_residual_kernel<<<gr, 256, 0, st>>>(c.W, c.ldw, (int)m, (int)n, c.r, c.U, c.V, c.sigma16, c.s, c.Rout, c.ldr);
  return true;
}

}  // namespace ptq
