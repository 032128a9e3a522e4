// What is stored for a layer and the form it is applied in (paper Sec. 3.2, Eq. 7; Sec. 3.4,
// Eq. 12; Algorithm 1, last lines; the time-complexity appendix):
//   * bit packing of the codes and its inverse with dequantization;
//   * the layer applied to a few tokens:  O = X~ Dequant(W_q)^T + ((X diag(s)^-1) V^T diag(sigma)) U,
//     X~ = X P Q  (the input is permuted and rotated once, the residual is never rotated back).
//
// Packing: 32 consecutive codes of a row (a chunk) form a little-endian bit stream of exactly d
// 32-bit words, code j in bits [j d, (j+1) d); the chunks are stored chunk-major,
// packed[chunk][row][d], and the grids group-major, scale[group][row] and zero[group][row], so
// that lanes that work on consecutive rows read consecutive memory.
//
// The product with the packed residual is bound by the rate at which the codes stream from
// memory (m n d / 8 bytes; the vectors and grids are a few percent of that).  A lane is a row;
// a workgroup takes 256 rows and a run of eight chunks (256 columns), whose piece of X~ it
// stages in LDS (all lanes read the same address: a broadcast), requests its eight chunks at
// once, and writes one partial sum per row and token; a second small kernel adds the partial
// sums of a row in a fixed order together with the low-rank part.  Splitting the columns rather
// than the rows keeps the staged piece of X~ tiny, so that the grid can be large enough to fill
// the chip without every workgroup re-reading all of X~.
#include "common.h"

namespace ptq {
namespace {

constexpr int kChunk = 32;   // codes per lane and step: d words

// Code j of a chunk from its d words; j and d are compile-time constants, so this is one
// bit-field extract, or two shifts and a mask where a 3-bit code straddles two words.
template <int BITS>
__device__ __forceinline__ uint32_t chunk_code(const uint32_t* __restrict__ words, int j) {
  const int pos = j * BITS, wi = pos >> 5, sh = pos & 31;
  constexpr uint32_t mask = (1u << BITS) - 1u;
  if (sh + BITS <= 32) return (words[wi] >> sh) & mask;
  return ((words[wi] >> sh) | (words[wi + 1] << (32 - sh))) & mask;
}

template <int BITS>
__device__ __forceinline__ void unpack_chunk(const uint32_t* __restrict__ words, uint8_t (&code)[kChunk]) {
#pragma unroll
  for (int j = 0; j < kChunk; ++j) code[j] = (uint8_t)chunk_code<BITS>(words, j);
}

template <int BITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ codes, int64_t ldc, int m, int n,
                                                   uint32_t* __restrict__ packed) {
  const int chunks = n / kChunk;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * chunks) return;
  const int c = (int)(e / m), row = (int)(e - (int64_t)c * m);   // rows fastest: the stores are contiguous
  const uint4* src = reinterpret_cast<const uint4*>(codes + (int64_t)row * ldc + c * kChunk);
  const uint4 lo = src[0], hi = src[1];
  const uint32_t raw[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  uint32_t* dst = packed + ((int64_t)c * m + row) * BITS;
  uint64_t acc = 0;
  int have = 0, w = 0;
#pragma unroll
  for (int j = 0; j < kChunk; ++j) {
    const uint32_t code = (raw[j >> 2] >> (8 * (j & 3))) & ((1u << BITS) - 1u);
    acc |= (uint64_t)code << have;
    have += BITS;
    if (have >= 32) {
      dst[w++] = (uint32_t)acc;
      acc >>= 32;
      have -= 32;
    }
  }
}

template <int BITS>
__global__ __launch_bounds__(256) void unpack_dequant_kernel(const uint32_t* __restrict__ packed, int m, int n,
                                                             const float* __restrict__ scales,
                                                             const uint8_t* __restrict__ zeros, int group,
                                                             double* __restrict__ Wq, int64_t ldq) {
  const int chunks = n / kChunk;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * chunks) return;
  const int c = (int)(e / m), row = (int)(e - (int64_t)c * m);
  const uint32_t* src = packed + ((int64_t)c * m + row) * BITS;
  uint32_t words[BITS];
#pragma unroll
  for (int w = 0; w < BITS; ++w) words[w] = src[w];
  uint8_t code[kChunk];
  unpack_chunk<BITS>(words, code);
  double* dst = Wq + (int64_t)row * ldq + c * kChunk;
#pragma unroll
  for (int j = 0; j < kChunk; ++j) {
    const int g = (c * kChunk + j) / group;   // a group may be as small as 16 columns
    const double sc = (double)scales[(int64_t)g * m + row];
    const double z = (double)zeros[(int64_t)g * m + row];
    dst[j] = sc * ((double)code[j] - z);
  }
}

// scale[row][group] -> scale[group][row], the same for the zero-points (32 x 32 tiles through LDS)
__global__ __launch_bounds__(256) void transpose_grids_kernel(const float* __restrict__ scales,
                                                              const uint8_t* __restrict__ zeros, int m, int ng,
                                                              float* __restrict__ scales_t,
                                                              uint8_t* __restrict__ zeros_t) {
  __shared__ float ts[32][33];
  __shared__ uint8_t tz[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int r0 = blockIdx.x * 32, g0 = blockIdx.y * 32;
  for (int k = ty; k < 32; k += 8) {
    const int row = r0 + k, g = g0 + tx;
    if (row < m && g < ng) { ts[k][tx] = scales[(int64_t)row * ng + g]; tz[k][tx] = zeros[(int64_t)row * ng + g]; }
  }
  __syncthreads();
  for (int k = ty; k < 32; k += 8) {
    const int g = g0 + k, row = r0 + tx;
    if (row < m && g < ng) { scales_t[(int64_t)g * m + row] = ts[tx][k]; zeros_t[(int64_t)g * m + row] = tz[tx][k]; }
  }
}

// ---- the layer applied to a few tokens ----------------------------------------------------
// Inputs prepared per call: X~ (float32, from the float64 rotation) and the low-rank
// coefficients  y[t][k] = sigma_k * sum_j V[k][j] x[t][j] / s[j].
__device__ __forceinline__ float e4m3_to_float(uint8_t c) {
  const int ef = (c >> 3) & 0xf, mt = c & 7;
  const float mag = ef == 0 ? ldexpf((float)mt, -9) : ldexpf((float)(8 + mt), ef - 10);
  return (c & 0x80) ? -mag : mag;
}
__device__ __forceinline__ float fp16_bits_to_float(uint16_t h) {
  const int ef = (h >> 10) & 31, mt = h & 0x3ff;
  float mag;
  if (ef == 31) mag = mt ? __builtin_nanf("") : __builtin_inff();
  else mag = ef == 0 ? ldexpf((float)mt, -24) : ldexpf((float)(1024 + mt), ef - 25);
  return (h & 0x8000) ? -mag : mag;
}

// one workgroup per (token, rank); the first also clears the counters of the product that follows
template <int DT>
__global__ __launch_bounds__(256) void low_rank_coeff_kernel(const void* __restrict__ X, int64_t ldx, int n,
                                                             const uint8_t* __restrict__ V,
                                                             const uint16_t* __restrict__ sigma,
                                                             const double* __restrict__ s, int r,
                                                             float* __restrict__ y, unsigned* __restrict__ done,
                                                             int counters) {
  if (blockIdx.x == 0)
    for (int i = threadIdx.x; i < counters; i += 256) done[i] = 0u;
  const int t = blockIdx.x / r, k = blockIdx.x - t * r;
  double acc = 0.0;
  for (int j = threadIdx.x; j < n; j += 256)
    acc += (double)e4m3_to_float(V[(int64_t)k * n + j]) * (load_as_f64<DT>(X, (int64_t)t * ldx + j) / s[j]);
  __shared__ double red[256];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) y[(int64_t)t * r + k] = (float)(red[0] * (double)fp16_bits_to_float(sigma[k]));
}

struct ForwardArgs {
  const uint32_t* packed;   // (n / 32) x m x BITS words
  const float* scales;      // n / group x m
  const uint8_t* zeros;     // n / group x m
  int m, n, group;
  const float* xt;          // tokens x n: X~
  const float* y;           // tokens x r
  const uint8_t* U;         // r x m, e4m3
  int r;
  float* partial;           // splits x B x m
  unsigned* done;           // one counter per block of 256 rows: zero on entry, left at zero
  float* O;                 // tokens x m
  int64_t ldo;
};

constexpr int kFwdRun = 8;   // chunks per workgroup: 256 columns

template <int BITS>
struct alignas(BITS == 3 ? 4 : (BITS == 2 ? 8 : 16)) Words { uint32_t w[BITS]; };

// grid: (row blocks of 256, runs of kFwdRun chunks); B tokens.  Requires group % 32 == 0.
template <int BITS, int B>
__global__ __launch_bounds__(256) void forward_partial_kernel(ForwardArgs a) {
  __shared__ float xs[B][kFwdRun * kChunk];
  __shared__ float xsum[B][kFwdRun];
  const int tid = threadIdx.x;
  const int m = a.m, n = a.n, chunks = n / kChunk;
  const int row = blockIdx.x * 256 + tid;
  const bool live = row < m;
  const int c0 = blockIdx.y * kFwdRun;
  const int nc = min(kFwdRun, chunks - c0);

  // the eight chunks of this row first: they are the long latency
  Words<BITS> wd[kFwdRun];
#pragma unroll
  for (int k = 0; k < kFwdRun; ++k) {
#pragma unroll
    for (int w = 0; w < BITS; ++w) wd[k].w[w] = 0u;
    if (live && k < nc) wd[k] = *reinterpret_cast<const Words<BITS>*>(a.packed + ((int64_t)(c0 + k) * m + row) * BITS);
  }
  // sum_j scale (code_j - zero) x_j = scale (sum_j code_j x_j - zero sum_j x_j): the second sum does
  // not depend on the row, so a weight costs an extract, a conversion and one multiply-add per token
  for (int e = tid; e < B * kFwdRun * (kChunk / 4); e += 256) {
    const int t = e / (kFwdRun * (kChunk / 4)), q = e - t * (kFwdRun * (kChunk / 4));   // q: float4 index in the run
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (q < nc * (kChunk / 4)) v = *reinterpret_cast<const float4*>(a.xt + (int64_t)t * n + c0 * kChunk + 4 * q);
    *reinterpret_cast<float4*>(&xs[t][4 * q]) = v;
    float sum = (v.x + v.y) + (v.z + v.w);     // eight consecutive threads hold one chunk
    sum += __shfl_xor(sum, 1);
    sum += __shfl_xor(sum, 2);
    sum += __shfl_xor(sum, 4);
    if ((q & 7) == 0) xsum[t][q >> 3] = sum;
  }
  __syncthreads();

  float acc[B];
#pragma unroll
  for (int t = 0; t < B; ++t) acc[t] = 0.f;
#pragma unroll
  for (int k = 0; k < kFwdRun; ++k) {
    if (k >= nc) break;
    const int g = (c0 + k) * kChunk / a.group;
    const float sc = live ? a.scales[(int64_t)g * m + row] : 0.f;
    const float z = live ? (float)a.zeros[(int64_t)g * m + row] : 0.f;
    float raw[B];
#pragma unroll
    for (int t = 0; t < B; ++t) raw[t] = 0.f;
#pragma unroll
    for (int q = 0; q < kChunk / 4; ++q) {
      float cf[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) cf[j] = (float)chunk_code<BITS>(wd[k].w, 4 * q + j);
#pragma unroll
      for (int t = 0; t < B; ++t) {
        const float4 x = *reinterpret_cast<const float4*>(&xs[t][k * kChunk + 4 * q]);
        raw[t] = fmaf(cf[3], x.w, fmaf(cf[2], x.z, fmaf(cf[1], x.y, fmaf(cf[0], x.x, raw[t]))));
      }
    }
#pragma unroll
    for (int t = 0; t < B; ++t) acc[t] = fmaf(sc, fmaf(-z, xsum[t][k], raw[t]), acc[t]);
  }
  // The partial sums go out device-coherently; the workgroup that counts itself last for its
  // block of rows adds the column runs in order, adds the low-rank part and writes the output:
  //   O[t][row] = sum over the column runs + sum_k U[k][row] y[t][k]
  if (live) {
#pragma unroll
    for (int t = 0; t < B; ++t)
      __hip_atomic_store(a.partial + ((int64_t)blockIdx.y * B + t) * m + row, acc[t], __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
  __shared__ int last;
  __builtin_amdgcn_s_waitcnt(0);   // every wave's stores acknowledged before the workgroup is counted
  __syncthreads();
  const int splits = gridDim.y;
  if (tid == 0) last = atomicAdd(a.done + blockIdx.x, 1u) + 1u == (unsigned)splits;
  __syncthreads();
  if (!last) return;
  if (tid == 0) __hip_atomic_store(a.done + blockIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (!live) return;
  float out[B];
#pragma unroll
  for (int t = 0; t < B; ++t) out[t] = 0.f;
  for (int sp0 = 0; sp0 < splits; sp0 += 8) {   // eight loads in flight per token, added in order
    float v[8][B];
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int t = 0; t < B; ++t) {
        const int sp = sp0 + k < splits ? sp0 + k : splits - 1;   // issued whatever sp: no branch, no wait
        v[k][t] = __hip_atomic_load(a.partial + ((int64_t)sp * B + t) * m + row, __ATOMIC_RELAXED,
                                    __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
    for (int k = 0; k < 8; ++k)
#pragma unroll
      for (int t = 0; t < B; ++t) out[t] += sp0 + k < splits ? v[k][t] : 0.f;
  }
  for (int k = 0; k < a.r; ++k) {
    const float u = e4m3_to_float(a.U[(int64_t)k * m + row]);
#pragma unroll
    for (int t = 0; t < B; ++t) out[t] = fmaf(u, a.y[(int64_t)t * a.r + k], out[t]);
  }
#pragma unroll
  for (int t = 0; t < B; ++t) a.O[(int64_t)t * a.ldo + row] = out[t];
}

__global__ void clear_counters_kernel(unsigned* done, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) done[i] = 0u;
}

// ---- many tokens: the same sums on the matrix cores ------------------------------------------
// With 8 or more tokens the row-per-lane kernel above is bound by feeding the same x to all lanes.
// Here a wave takes 32 rows and up to 32 tokens and accumulates  raw[row][t] = sum_j code_j x_tj
// with the float32 32 x 32 x 2 MFMA (full float32 products and sums): lane l supplies the code of
// row l % 32 for the column of parity l / 32 -- both halves of the wave load the same packed
// words and extract alternate codes, so nothing is transposed -- and x[t = l % 32] of that
// column from LDS.  At the end of a quantization group (or of the run of 8 chunks) the 16
// accumulators of a lane get  scale (raw - zero sum_j x_tj)  for their rows and start again.
// grid: (row blocks of 128, runs of kFwdRun chunks), 4 waves; the partial sums are added by the kernel below.
constexpr int kMfmaTokens = 32, kMfmaRows = 128;

template <int BITS>
__global__ __launch_bounds__(256) void forward_mfma_kernel(ForwardArgs a, int tokens) {
  __shared__ float xs[kFwdRun * kChunk][kMfmaTokens + 1];   // [column of the run][token]; the odd pitch spreads the transposing stores over the banks
  __shared__ float xsum[kFwdRun][kMfmaTokens];
  __shared__ float gsc[kFwdRun][kMfmaRows], gz[kFwdRun][kMfmaRows];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int m = a.m, n = a.n, chunks = n / kChunk;
  const int c0 = blockIdx.y * kFwdRun;
  const int nc = min(kFwdRun, chunks - c0);
  const int row = blockIdx.x * kMfmaRows + w * 32 + (lane & 31);   // the row whose codes this lane supplies
  const int parity = lane >> 5;
  const bool live = row < m;

  Words<BITS> wd[kFwdRun];
#pragma unroll
  for (int k = 0; k < kFwdRun; ++k) {
#pragma unroll
    for (int q = 0; q < BITS; ++q) wd[k].w[q] = 0u;
    if (live && k < nc) wd[k] = *reinterpret_cast<const Words<BITS>*>(a.packed + ((int64_t)(c0 + k) * m + row) * BITS);
  }
  // x of the run, transposed to [column][token] (zeros past the last token and the last chunk):
  // eight 16-byte loads per thread, all requested before the first is stored
  {
    constexpr int kQuads = kFwdRun * kChunk / 4;   // per token
    float4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = tid + 256 * i, t = e / kQuads, c = 4 * (e - t * kQuads);
      const bool ok = t < tokens && c < nc * kChunk;
      const float4 x = *reinterpret_cast<const float4*>(a.xt + (int64_t)(t < tokens ? t : 0) * n + c0 * kChunk +
                                                         (c < nc * kChunk ? c : 0));
      v[i] = ok ? x : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int e = tid + 256 * i, t = e / kQuads, c = 4 * (e - t * kQuads);
      xs[c][t] = v[i].x; xs[c + 1][t] = v[i].y; xs[c + 2][t] = v[i].z; xs[c + 3][t] = v[i].w;
      float sum = (v[i].x + v[i].y) + (v[i].z + v[i].w);   // eight consecutive lanes hold one chunk of a token
      sum += __shfl_xor(sum, 1);
      sum += __shfl_xor(sum, 2);
      sum += __shfl_xor(sum, 4);
      if ((c & (kChunk - 1)) == 0) xsum[c / kChunk][t] = sum;
    }
  }
  // scale and zero of each chunk's group for the block's 128 rows
  for (int e = tid; e < kFwdRun * kMfmaRows; e += 256) {
    const int k = e / kMfmaRows, rl = e - k * kMfmaRows;
    const int orow = blockIdx.x * kMfmaRows + rl;
    const bool ok = k < nc && orow < m;
    const int g = ((c0 + (k < nc ? k : 0)) * kChunk) / a.group;
    gsc[k][rl] = ok ? a.scales[(int64_t)g * m + orow] : 0.f;
    gz[k][rl] = ok ? (float)a.zeros[(int64_t)g * m + orow] : 0.f;
  }
  __syncthreads();

  // accumulator r of a lane is row (r / 4) * 8 + (lane / 32) * 4 + r % 4 of the wave's 32, token lane % 32
  const int t_out = lane & 31;
  f32x16 acc, total;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[r] = 0.f; total[r] = 0.f; }
  float xsg = 0.f;
#pragma unroll
  for (int k = 0; k < kFwdRun; ++k) {
    if (k >= nc) break;
    float xv[kChunk / 2];   // the chunk's x values first: one LDS latency per chunk, not per MFMA
#pragma unroll
    for (int i = 0; i < kChunk / 2; ++i) xv[i] = xs[k * kChunk + 2 * i + parity][t_out];
#pragma unroll
    for (int i = 0; i < kChunk / 2; ++i) {
      const uint32_t ce = chunk_code<BITS>(wd[k].w, 2 * i), co = chunk_code<BITS>(wd[k].w, 2 * i + 1);
      const float cf = (float)(parity ? co : ce);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(cf, xv[i], acc, 0, 0, 0);
    }
    xsg += xsum[k][t_out];
    const int col_end = (c0 + k + 1) * kChunk;
    if (col_end % a.group == 0 || k == nc - 1) {   // the group ends here, or the run does
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = w * 32 + (r >> 2) * 8 + parity * 4 + (r & 3);
        total[r] = fmaf(gsc[k][rl], fmaf(-gz[k][rl], xsg, acc[r]), total[r]);
        acc[r] = 0.f;
      }
      xsg = 0.f;
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int orow = blockIdx.x * kMfmaRows + w * 32 + (r >> 2) * 8 + parity * 4 + (r & 3);
    if (orow < m && t_out < tokens) a.partial[((int64_t)blockIdx.y * kMfmaTokens + t_out) * m + orow] = total[r];
  }
}

// O[t][row] = sum over the column runs, in order, + sum_k U[k][row] y[t][k] for the matrix-core
// passes: with up to 32 tokens the sums are enough work for a launch of their own over the whole
// chip (done by the last workgroup of each row block they took longer than the products).
// grid: (rows / 256, groups of four tokens)
__global__ __launch_bounds__(256) void forward_mfma_finish_kernel(ForwardArgs a, int tokens, int splits) {
  const int row = blockIdx.x * 256 + threadIdx.x;
  const int t0 = blockIdx.y * 4;
  if (row >= a.m) return;
  float out[4] = {0.f, 0.f, 0.f, 0.f};
  for (int sp0 = 0; sp0 < splits; sp0 += 16) {
    float v[16][4];
#pragma unroll
    for (int k = 0; k < 16; ++k)
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int sp = sp0 + k < splits ? sp0 + k : splits - 1;   // issued whatever sp: no branch, no wait
        const int tt = t0 + t < tokens ? t0 + t : tokens - 1;
        v[k][t] = a.partial[((int64_t)sp * kMfmaTokens + tt) * a.m + row];
      }
#pragma unroll
    for (int k = 0; k < 16; ++k)
#pragma unroll
      for (int t = 0; t < 4; ++t) out[t] += sp0 + k < splits ? v[k][t] : 0.f;
  }
  for (int k = 0; k < a.r; ++k) {
    const float u = e4m3_to_float(a.U[(int64_t)k * a.m + row]);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      if (t0 + t < tokens) out[t] = fmaf(u, a.y[(int64_t)(t0 + t) * a.r + k], out[t]);
  }
#pragma unroll
  for (int t = 0; t < 4; ++t)
    if (t0 + t < tokens) a.O[(int64_t)(t0 + t) * a.ldo + row] = out[t];
}

template <int BITS>
void launch_forward_mfma(const ForwardArgs& a, int tokens, hipStream_t st) {
  const int splits = (int)ceil_div(a.n / kChunk, kFwdRun);
  dim3 g((unsigned)ceil_div(a.m, kMfmaRows), (unsigned)splits);
  forward_mfma_kernel<BITS><<<g, 256, 0, st>>>(a, tokens);
  dim3 gf((unsigned)ceil_div(a.m, 256), (unsigned)ceil_div(tokens, 4));
  forward_mfma_finish_kernel<<<gf, 256, 0, st>>>(a, tokens, splits);
}

template <int BITS, int B>
void launch_forward_b(const ForwardArgs& a, hipStream_t st) {
  const int splits = (int)ceil_div(a.n / kChunk, kFwdRun);
  dim3 g((unsigned)ceil_div(a.m, 256), (unsigned)splits);
  forward_partial_kernel<BITS, B><<<g, 256, 0, st>>>(a);
}

// up to 32 tokens per pass over the codes on the matrix cores while 8 or more are left, then
// four, two or one token per pass
template <int BITS>
void launch_forward(const ForwardArgs& a, int tokens, hipStream_t st) {
  ForwardArgs b = a;
  int done = 0;
  while (done < tokens) {
    const int left = tokens - done;
    int step;
    if (left >= 8) { step = left < kMfmaTokens ? left : kMfmaTokens; launch_forward_mfma<BITS>(b, step, st); }
    else if (left >= 4) { step = 4; launch_forward_b<BITS, 4>(b, st); }
    else if (left >= 2) { step = 2; launch_forward_b<BITS, 2>(b, st); }
    else { step = 1; launch_forward_b<BITS, 1>(b, st); }
    done += step;
    b.xt = a.xt + (int64_t)done * a.n;
    b.y = a.y + (int64_t)done * a.r;
    b.O = a.O + (int64_t)done * a.ldo;
  }
}

}  // namespace

ptq_status pack_grids_launch(const float* scales, const uint8_t* zeros, int64_t m, int64_t ng, float* scales_t,
                             uint8_t* zeros_t, hipStream_t st) {
  dim3 g((unsigned)ceil_div(m, 32), (unsigned)ceil_div(ng, 32));
  transpose_grids_kernel<<<g, 256, 0, st>>>(scales, zeros, (int)m, (int)ng, scales_t, zeros_t);
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status pack_codes_launch(const uint8_t* codes, int64_t ldc, int64_t m, int64_t n, int bits, uint32_t* packed,
                             hipStream_t st) {
  const unsigned grid = (unsigned)ceil_div(m * (n / kChunk), 256);
  switch (bits) {
    case 2: pack_kernel<2><<<grid, 256, 0, st>>>(codes, ldc, (int)m, (int)n, packed); break;
    case 3: pack_kernel<3><<<grid, 256, 0, st>>>(codes, ldc, (int)m, (int)n, packed); break;
    case 4: pack_kernel<4><<<grid, 256, 0, st>>>(codes, ldc, (int)m, (int)n, packed); break;
    case 8: pack_kernel<8><<<grid, 256, 0, st>>>(codes, ldc, (int)m, (int)n, packed); break;
    default: return PTQ_ERR_ARG;
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

ptq_status unpack_dequant_launch(const uint32_t* packed, int64_t m, int64_t n, int bits, const float* scales,
                                 const uint8_t* zeros, int group, double* Wq, int64_t ldq, hipStream_t st) {
  const unsigned grid = (unsigned)ceil_div(m * (n / kChunk), 256);
  switch (bits) {
    case 2: unpack_dequant_kernel<2><<<grid, 256, 0, st>>>(packed, (int)m, (int)n, scales, zeros, group, Wq, ldq); break;
    case 3: unpack_dequant_kernel<3><<<grid, 256, 0, st>>>(packed, (int)m, (int)n, scales, zeros, group, Wq, ldq); break;
    case 4: unpack_dequant_kernel<4><<<grid, 256, 0, st>>>(packed, (int)m, (int)n, scales, zeros, group, Wq, ldq); break;
    case 8: unpack_dequant_kernel<8><<<grid, 256, 0, st>>>(packed, (int)m, (int)n, scales, zeros, group, Wq, ldq); break;
    default: return PTQ_ERR_ARG;
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

static size_t forward_partial_bytes(int64_t m, int64_t n) {
  return align_up((size_t)ceil_div(n / kChunk, kFwdRun) * kMfmaTokens * (size_t)m * sizeof(float), 256);
}

static size_t forward_counter_bytes(int64_t m) { return align_up((size_t)ceil_div(m, 256) * sizeof(unsigned), 256); }

// ---- scratch for callers that cannot allocate -----------------------------------------------
// One array per GPU, part of the library's code object: the device memory the forward call needs
// beyond its inputs and outputs (the rotated input, the low-rank coefficients, the partial sums of
// the column runs and the row-block counters).  Its name is a host-side stand-in, not a device
// address: the address on the current device comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

size_t linear_forward_static_scratch_bytes() { return kStaticScratchBytes; }

ptq_status linear_forward_static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> per_device[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PTQ_ERR_HIP;
  void* p = per_device[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PTQ_ERR_HIP;
    per_device[dev].store(p, std::memory_order_release);   // every thread gets the same address: no race
  }
  *ptr = p;
  return PTQ_OK;
}

size_t linear_forward_workspace_bytes(int64_t tokens, int64_t m, int64_t n, int64_t r) {
  return align_up((size_t)tokens * n * sizeof(float), 256) +
         align_up((size_t)tokens * (r > 0 ? r : 1) * sizeof(float), 256) + forward_partial_bytes(m, n) +
         forward_counter_bytes(m);
}

ptq_status linear_forward_launch(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m, int64_t n,
                                 const uint32_t* packed, int bits, const float* scales, const uint8_t* zeros,
                                 int group, const int32_t* perm, int b_I, int b_H, const uint8_t* U,
                                 const uint8_t* V, const uint16_t* sigma, int r, const double* s, float* O,
                                 int64_t ldo, void* ws, hipStream_t st) {
  char* base = static_cast<char*>(ws);
  float* xt = reinterpret_cast<float*>(base);
  float* y = reinterpret_cast<float*>(reinterpret_cast<char*>(xt) + align_up((size_t)tokens * n * sizeof(float), 256));
  float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(y) +
                                            align_up((size_t)tokens * (r > 0 ? r : 1) * sizeof(float), 256));
  unsigned* done = reinterpret_cast<unsigned*>(reinterpret_cast<char*>(partial) + forward_partial_bytes(m, n));
  // X~ = X P Q: the rows of X go through the same transform as the rows of the residual
  ptq_status rc = lopro_rotate_input_launch(X, xdt, ldx, tokens, n, perm, b_I, b_H, xt, n, st);
  if (rc != PTQ_OK) return rc;
  const int counters = (int)ceil_div(m, 256);
  if (r > 0) {
    const unsigned g = (unsigned)(tokens * r);
    switch (xdt) {
      case PTQ_F32: low_rank_coeff_kernel<PTQ_F32><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y, done, counters); break;
      case PTQ_BF16: low_rank_coeff_kernel<PTQ_BF16><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y, done, counters); break;
      case PTQ_F64: low_rank_coeff_kernel<PTQ_F64><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y, done, counters); break;
      default: return PTQ_ERR_DTYPE;
    }
  } else {
    clear_counters_kernel<<<(unsigned)ceil_div(counters, 256), 256, 0, st>>>(done, counters);
  }
  ForwardArgs a{packed, scales, zeros, (int)m, (int)n, group, xt, y, U, r, partial, done, O, ldo};
  switch (bits) {
    case 2: launch_forward<2>(a, (int)tokens, st); break;
    case 3: launch_forward<3>(a, (int)tokens, st); break;
    case 4: launch_forward<4>(a, (int)tokens, st); break;
    case 8: launch_forward<8>(a, (int)tokens, st); break;
    default: return PTQ_ERR_ARG;
  }
  PTQ_HIP_CHECK_LAUNCH();
  return PTQ_OK;
}

}  // namespace ptq
