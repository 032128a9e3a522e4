// Diagnostic probe, built into its own small library (libptq_probe.so) and used by bench.py's
// --mfma-control only: what the matrix cores of this chip sustain when nothing but MFMAs is issued from
// registers -- the ceiling the product kernels are measured against -- with benign operands (all lanes
// the same few values) and with random operand bits (the data dependence of the power limit).
// kind 0: bf16 32x32x16 (16 accumulator tiles per wave, the Hessian kernel's shape), kind 1: float64
// 16x16x4 (8 accumulator tiles per wave).  One wave per SIMD, `blocks` workgroups of 256 threads.
// The file is compiled twice: as it is (the compiler then keeps MFMA accumulators in AGPRs), exporting
// ptq_probe_mfma, and with -DPTQ_PROBE_VGPR_FORM and the option that keeps them in ordinary VGPRs,
// exporting ptq_probe_mfma_vgpr.  For float64 the two forms sustain different rates.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {
typedef __attribute__((__vector_size__(4 * sizeof(double)))) double f64x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// clk[0] = ticks of the constant 100 MHz counter, clk[1] = shader clock cycles, both over the loop of
// workgroup 0, wave 0
__global__ __launch_bounds__(256) void probe_bf16(float* out, long long* clk, int iters, int random_bits) {
  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
  bf16x8 fa[4], fb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    u32x4 ua, ub;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // random: bfloat16 values with random sign and mantissa, exponents spread over a few binades
      // (activations-like); benign: the value 1.0 everywhere
      const uint32_t ha = mix(threadIdx.x * 977u + i * 131u + w * 17u + 1u), hb = mix(ha + 0x9e3779b9u);
      ua[w] = random_bits ? ((ha & 0x807f807fu) | 0x3e003e00u | ((ha >> 3) & 0x01800180u)) : 0x3f803f80u;
      ub[w] = random_bits ? ((hb & 0x807f807fu) | 0x3e003e00u | ((hb >> 3) & 0x01800180u)) : 0x3f803f80u;
    }
    fa[i] = __builtin_bit_cast(bf16x8, ua);
    fb[i] = __builtin_bit_cast(bf16x8, ub);
  }
  const long long w0 = wall_clock64(), c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
  }
  const long long w1 = wall_clock64(), c1 = clock64();
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[a][b][r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk[0] = w1 - w0;
    clk[1] = c1 - c0;
  }
}

__global__ __launch_bounds__(256) void probe_f64(float* out, long long* clk, int iters, int random_bits) {
  f64x4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f64x4{0, 0, 0, 0};
  double a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t h = mix(threadIdx.x * 977u + i * 131u + 7u), h2 = mix(h + 0x9e3779b9u);
    a[i] = random_bits ? ((double)(int)h * 0x1p-31 + (double)h2 * 0x1p-63) : 1.0000001;
    b[i] = random_bits ? ((double)(int)h2 * 0x1p-31 + (double)h * 0x1p-64) : 0.9999999;
  }
  const long long w0 = wall_clock64(), c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u & 3], b[(u >> 1) & 3], acc[u], 0, 0, 0);
  }
  const long long w1 = wall_clock64(), c1 = clock64();
  double s = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  out[blockIdx.x * 256 + threadIdx.x] = (float)s;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clk[0] = w1 - w0;
    clk[1] = c1 - c0;
  }
}

}  // namespace

#ifdef PTQ_PROBE_VGPR_FORM
#define PTQ_PROBE_ENTRY ptq_probe_mfma_vgpr
#else
#define PTQ_PROBE_ENTRY ptq_probe_mfma
#endif

extern "C" {
// out: blocks * 256 floats, clk: 2 int64, both device memory of the caller.  Returns the number of
// floating-point operations the launch executes (0 on a bad argument); enqueues on `stream`.
double PTQ_PROBE_ENTRY(int kind, int random_bits, int iters, int blocks, float* out, long long* clk, void* stream) {
  if (!out || !clk || iters <= 0 || blocks <= 0) return 0.0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (kind == 0) {
    probe_bf16<<<blocks, 256, 0, st>>>(out, clk, iters, random_bits);
    return (double)blocks * 4.0 * iters * 16.0 * 32768.0;
  }
  if (kind == 1) {
    probe_f64<<<blocks, 256, 0, st>>>(out, clk, iters, random_bits);
    return (double)blocks * 4.0 * iters * 8.0 * 2048.0;
  }
  return 0.0;
}
}
