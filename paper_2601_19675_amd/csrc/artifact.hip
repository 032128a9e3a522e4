// What is stored for a layer and the form it is applied in (paper Sec. 3.2, Eq. 7; Sec. 3.4,
// Eq. 12; Algorithm 1, last lines; the time-complexity appendix):
//   * bit packing of the codes and its inverse with dequantization;
//   * the layer applied to a few tokens:  O = X~ Dequant(W_q)^T + ((X diag(s)^-1) V^T diag(sigma)) U,
//     X~ = X P Q  (the input is permuted and rotated once, the residual is never rotated back).
//
// Packing: code j of a row occupies bits [j d, (j+1) d) of the row's bit stream, stored in
// little-endian 32-bit words; 32 codes fill exactly d words, which is the unit a lane works on.
//
// The product with the packed residual is bound by the rate at which the codes stream from
// memory (m n d / 8 bytes; the vectors and grids are a few percent of that).  A wave takes a
// few rows; each lane takes 32-column chunks, keeps that chunk of X~ for all tokens in
// registers and reuses it for the wave's rows, so that nothing but the codes is read per row.
#include "common.h"

namespace ptq {
namespace {

constexpr int kChunk = 32;   // codes per lane and step: d words

// The 32 codes of a chunk from its d words.
template <int BITS>
__device__ __forceinline__ void unpack_chunk(const uint32_t* __restrict__ words, uint8_t (&code)[kChunk]) {
  uint64_t acc = 0;
  int have = 0, w = 0;
#pragma unroll
  for (int j = 0; j < kChunk; ++j) {
    if (have < BITS) {
      acc |= (uint64_t)words[w++] << have;
      have += 32;
    }
    code[j] = (uint8_t)(acc & ((1u << BITS) - 1u));
    acc >>= BITS;
    have -= BITS;
  }
}

template <int BITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ codes, int64_t ldc, int m, int n,
                                                   uint32_t* __restrict__ packed) {
  const int chunks = n / kChunk;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= (int64_t)m * chunks) return;
  const int row = (int)(e / chunks), c = (int)(e - (int64_t)row * chunks);
  const uint4* src = reinterpret_cast<const uint4*>(codes + (int64_t)row * ldc + c * kChunk);
  const uint4 lo = src[0], hi = src[1];
  const uint32_t raw[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  uint32_t* dst = packed + ((int64_t)row * chunks + c) * BITS;
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
  const int row = (int)(e / chunks), c = (int)(e - (int64_t)row * chunks);
  const uint32_t* src = packed + ((int64_t)row * chunks + c) * BITS;
  uint32_t words[BITS];
#pragma unroll
  for (int w = 0; w < BITS; ++w) words[w] = src[w];
  uint8_t code[kChunk];
  unpack_chunk<BITS>(words, code);
  const int ng = n / group;
  double* dst = Wq + (int64_t)row * ldq + c * kChunk;
#pragma unroll
  for (int j = 0; j < kChunk; ++j) {
    const int g = (c * kChunk + j) / group;   // a group may be as small as 16 columns
    const double sc = (double)scales[(int64_t)row * ng + g];
    const double z = (double)zeros[(int64_t)row * ng + g];
    dst[j] = sc * ((double)code[j] - z);
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

__global__ __launch_bounds__(256) void narrow_kernel(const double* __restrict__ in, int64_t count,
                                                     float* __restrict__ out) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e < count) out[e] = (float)in[e];
}

// one workgroup per (token, rank)
template <int DT>
__global__ __launch_bounds__(256) void low_rank_coeff_kernel(const void* __restrict__ X, int64_t ldx, int n,
                                                             const uint8_t* __restrict__ V,
                                                             const uint16_t* __restrict__ sigma,
                                                             const double* __restrict__ s, int r,
                                                             float* __restrict__ y) {
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
  const uint32_t* packed;   // m x (n / 32) x BITS words
  const float* scales;      // m x n / group
  const uint8_t* zeros;     // m x n / group
  int m, n, group;
  const float* xt;          // tokens x n: X~
  const float* y;           // tokens x r
  const uint8_t* U;         // r x m, e4m3
  int r;
  float* O;                 // tokens x m
  int64_t ldo;
};

constexpr int kFwdWaves = 4;
constexpr int kFwdRows = 4;   // rows of W per wave

// B tokens per launch.  A lane's chunks are c = lane, lane + 64, ...; requires group % 32 == 0.
template <int BITS, int B>
__global__ __launch_bounds__(64 * kFwdWaves) void forward_kernel(ForwardArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int row0 = (blockIdx.x * kFwdWaves + wave) * kFwdRows;
  if (row0 >= a.m) return;
  const int chunks = a.n / kChunk, ng = a.n / a.group;
  float acc[kFwdRows][B];
#pragma unroll
  for (int i = 0; i < kFwdRows; ++i)
#pragma unroll
    for (int t = 0; t < B; ++t) acc[i][t] = 0.f;

  for (int c = lane; c < chunks; c += 64) {
    float x[B][kChunk];
#pragma unroll
    for (int t = 0; t < B; ++t) {
      const float4* px = reinterpret_cast<const float4*>(a.xt + (int64_t)t * a.n + c * kChunk);
#pragma unroll
      for (int q = 0; q < kChunk / 4; ++q) {
        const float4 v = px[q];
        x[t][4 * q] = v.x; x[t][4 * q + 1] = v.y; x[t][4 * q + 2] = v.z; x[t][4 * q + 3] = v.w;
      }
    }
    const int g = c * kChunk / a.group;
#pragma unroll
    for (int i = 0; i < kFwdRows; ++i) {
      const int row = row0 + i;
      if (row >= a.m) break;
      const uint32_t* src = a.packed + ((int64_t)row * chunks + c) * BITS;
      uint32_t words[BITS];
#pragma unroll
      for (int w = 0; w < BITS; ++w) words[w] = src[w];
      uint8_t code[kChunk];
      unpack_chunk<BITS>(words, code);
      const float sc = a.scales[(int64_t)row * ng + g];
      const float z = (float)a.zeros[(int64_t)row * ng + g];
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const float wq = sc * ((float)code[j] - z);
#pragma unroll
        for (int t = 0; t < B; ++t) acc[i][t] = fmaf(wq, x[t][j], acc[i][t]);
      }
    }
  }
  // the low-rank part rides on the same reduction: lane k adds  U[k][row] * y[t][k]
#pragma unroll
  for (int i = 0; i < kFwdRows; ++i) {
    const int row = row0 + i;
    if (row >= a.m) break;
    for (int k = lane; k < a.r; k += 64) {
      const float u = e4m3_to_float(a.U[(int64_t)k * a.m + row]);
#pragma unroll
      for (int t = 0; t < B; ++t) acc[i][t] = fmaf(u, a.y[(int64_t)t * a.r + k], acc[i][t]);
    }
#pragma unroll
    for (int t = 0; t < B; ++t) {
      float v = acc[i][t];
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
      if (lane == 0) a.O[(int64_t)t * a.ldo + row] = v;
    }
  }
}

template <int BITS>
void launch_forward(const ForwardArgs& a, int tokens, hipStream_t st) {
  const unsigned grid = (unsigned)ceil_div(a.m, kFwdWaves * kFwdRows);
  ForwardArgs b = a;
  int done = 0;
  while (done < tokens) {
    const int left = tokens - done;
    if (left >= 4) {
      forward_kernel<BITS, 4><<<grid, 64 * kFwdWaves, 0, st>>>(b);
      done += 4;
    } else if (left >= 2) {
      forward_kernel<BITS, 2><<<grid, 64 * kFwdWaves, 0, st>>>(b);
      done += 2;
    } else {
      forward_kernel<BITS, 1><<<grid, 64 * kFwdWaves, 0, st>>>(b);
      done += 1;
    }
    b.xt = a.xt + (int64_t)done * a.n;
    b.y = a.y + (int64_t)done * a.r;
    b.O = a.O + (int64_t)done * a.ldo;
  }
}

}  // namespace

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

size_t linear_forward_workspace_bytes(int64_t tokens, int64_t n, int64_t r) {
  return align_up((size_t)tokens * n * sizeof(double), 256) + align_up((size_t)tokens * n * sizeof(float), 256) +
         align_up((size_t)tokens * (r > 0 ? r : 1) * sizeof(float), 256);
}

ptq_status linear_forward_launch(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m, int64_t n,
                                 const uint32_t* packed, int bits, const float* scales, const uint8_t* zeros,
                                 int group, const int32_t* perm, int b_I, int b_H, const uint8_t* U,
                                 const uint8_t* V, const uint16_t* sigma, int r, const double* s, float* O,
                                 int64_t ldo, void* ws, hipStream_t st) {
  char* base = static_cast<char*>(ws);
  double* xt64 = reinterpret_cast<double*>(base);
  float* xt = reinterpret_cast<float*>(base + align_up((size_t)tokens * n * sizeof(double), 256));
  float* y = reinterpret_cast<float*>(reinterpret_cast<char*>(xt) + align_up((size_t)tokens * n * sizeof(float), 256));
  // X~ = X P Q: the rows of X go through the same transform as the rows of the residual
  ptq_status rc = lopro_rotate_weight_launch(X, xdt, ldx, tokens, n, perm, b_I, b_H, xt64, n, st);
  if (rc != PTQ_OK) return rc;
  narrow_kernel<<<(unsigned)ceil_div(tokens * n, 256), 256, 0, st>>>(xt64, tokens * n, xt);
  if (r > 0) {
    const unsigned g = (unsigned)(tokens * r);
    switch (xdt) {
      case PTQ_F32: low_rank_coeff_kernel<PTQ_F32><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y); break;
      case PTQ_BF16: low_rank_coeff_kernel<PTQ_BF16><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y); break;
      case PTQ_F64: low_rank_coeff_kernel<PTQ_F64><<<g, 256, 0, st>>>(X, ldx, (int)n, V, sigma, s, r, y); break;
      default: return PTQ_ERR_DTYPE;
    }
  }
  ForwardArgs a{packed, scales, zeros, (int)m, (int)n, group, xt, y, U, r, O, ldo};
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
