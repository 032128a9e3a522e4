// Shared declarations for the gfx950 kernels of libptq (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include "../../include/ptq.h"

namespace ptq {

typedef __attribute__((__vector_size__(4 * sizeof(double)))) double f64x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Element of a stored weight / activation matrix widened exactly to float64.
template <int DT>
__device__ __forceinline__ double load_as_f64(const void* p, int64_t idx) {
  if constexpr (DT == PTQ_F32) {
    return static_cast<double>(static_cast<const float*>(p)[idx]);
  } else if constexpr (DT == PTQ_BF16) {
    return static_cast<double>(bf16_bits_to_f32(static_cast<const uint16_t*>(p)[idx]));
  } else {
    return static_cast<const double*>(p)[idx];
  }
}

// The same in two steps, so that a kernel can keep the raw stored value in a
// register while the load is in flight and widen it only when it is consumed.
template <int DT> struct StoredType { using type = double; };
template <> struct StoredType<PTQ_F32> { using type = float; };
template <> struct StoredType<PTQ_BF16> { using type = uint16_t; };
template <int DT>
__device__ __forceinline__ typename StoredType<DT>::type load_stored(const void* p, int64_t idx) {
  return static_cast<const typename StoredType<DT>::type*>(p)[idx];
}
template <int DT>
__device__ __forceinline__ double stored_to_f64(typename StoredType<DT>::type v) {
  if constexpr (DT == PTQ_BF16) return static_cast<double>(bf16_bits_to_f32(v));
  else return static_cast<double>(v);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t align_up(size_t a, size_t b) { return (a + b - 1) / b * b; }

// Lets `Kernel` use up to `bytes` of dynamic LDS (more than the 64 KB default needs the
// attribute).  Done once per kernel and device; safe to call from several host threads.
template <auto Kernel>
inline bool lds_opt_in(int bytes) {
  static std::atomic<uint64_t> done{0};  // one bit per device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  const uint64_t bit = uint64_t{1} << (dev & 63);
  if (done.load(std::memory_order_acquire) & bit) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          bytes) != hipSuccess)
    return false;
  done.fetch_or(bit, std::memory_order_release);
  return true;
}

// Lane exchanges inside a row of 16 lanes by data-parallel primitives: register moves, no trip
// through the LDS crossbar (which a shuffle of a float64 makes twice).  Applied in this order --
// pairs, half quads, half mirror, mirror -- with an associative, commutative operation after
// each, every lane ends up with the result over 2, 4, 8, 16 lanes.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const unsigned long long bits = __double_as_longlong(v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)bits, CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(bits >> 32), CTRL, 0xf, 0xf, false);
  return __longlong_as_double((long long)(((unsigned long long)(unsigned)hi << 32) | (unsigned)lo));
}
constexpr int kDppSwapPairs = 0xB1;      // quad_perm [1, 0, 3, 2]
constexpr int kDppSwapHalfQuads = 0x4E;  // quad_perm [2, 3, 0, 1]
constexpr int kDppHalfMirror = 0x141;    // lane i of 8 <- lane 7 - i
constexpr int kDppMirror = 0x140;        // lane i of 16 <- lane 15 - i

#define PTQ_HIP_CHECK_LAUNCH()                         \
  do {                                                 \
    if (hipGetLastError() != hipSuccess) return PTQ_ERR_HIP; \
  } while (0)

// ---- per-op host entry points (defined in the .hip files) -------------------
size_t hessian_workspace_bytes(int64_t n, int64_t t);
ptq_status hessian_launch(double* H, int64_t ldh, const void* X, ptq_dtype xdt, int64_t t, int64_t n,
                          int64_t ldx, void* ws, size_t ws_bytes, hipStream_t s);

// main kernel of the float32 case (hessian_f32.hip): float64 partial tiles of 64 or 128 channels squared
bool hessian_f32_partials_launch(const float* X, int64_t ldx, int64_t t, int n, int64_t tok0, int chunk, int ntb,
                                 int tile, dim3 grid, double* partial, hipStream_t s);

size_t cholesky_workspace_bytes(int64_t n);
ptq_status cholesky_launch(const double* H, int64_t ldh, int64_t n, double damp, double* U,
                           int64_t ldu, uint8_t* dead_mask, int32_t* info, void* ws, size_t ws_bytes,
                           hipStream_t s);

size_t quantize_workspace_bytes(int64_t m, int64_t n);
ptq_status quantize_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                           const double* U, int64_t ldu, const uint8_t* dead_mask, int bits, int group,
                           int block, uint8_t* codes, float* scales, uint8_t* zeros, double* Wq,
                           double* row_err2, int static_groups, void* ws, size_t ws_bytes, hipStream_t s);

ptq_status quantize_vq_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* U,
                              int64_t ldu, const uint8_t* dead_mask, const float* codebook, int entries, int dim,
                              int block, uint8_t* indices, double* Wq, double* row_err2, void* ws, size_t ws_bytes,
                              hipStream_t s);

size_t layer_error_workspace_bytes(int64_t m, int64_t n);
ptq_status layer_error_launch(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                              int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                              size_t ws_bytes, hipStream_t s);


size_t lopro_order_workspace_bytes(int64_t n);
size_t lopro_hessian_workspace_bytes(int64_t n);
ptq_status lopro_order_launch(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n, const double* H,
                              int64_t ldh, int descending, int32_t* perm, double* keys, void* ws,
                              hipStream_t s);
ptq_status lopro_rotate_weight_launch(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                      const int32_t* perm, int b_I, int b_H, double* Rout, int64_t ldo,
                                      hipStream_t s);
// the same transform on the rows of X, written as float32: the input of the stored layer's product
ptq_status lopro_rotate_input_launch(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t n,
                                     const int32_t* perm, int b_I, int b_H, float* Xout, int64_t ldo,
                                     hipStream_t st);
ptq_status lopro_unrotate_weight_launch(const double* Rq, int64_t ldq, int64_t m, int64_t n,
                                        const int32_t* perm, int b_I, int b_H, double* Wout, int64_t ldo,
                                        hipStream_t s);
ptq_status lopro_rotate_hessian_launch(const double* H, int64_t ldh, int64_t n, const int32_t* perm, int b_I,
                                       int b_H, double* Hout, int64_t ldo, void* ws, hipStream_t s);


size_t abs_sum_workspace_bytes(int64_t n);
ptq_status abs_sum_launch(double* asum, const void* X, ptq_dtype xdt, int64_t t, int64_t n, int64_t ldx, void* ws,
                          hipStream_t s);
ptq_status activation_scale_launch(const double* asum, int64_t tokens, int64_t n, double* s, hipStream_t st);
size_t r1svd_workspace_bytes(int64_t m, int64_t n);
int64_t r1svd_max_columns();
void r1svd_select(int launch_form, long long spin_limit);
ptq_status r1svd_launch(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* s,
                        const float* S, int64_t lds, int r, int it, uint8_t* U, uint8_t* V, uint16_t* sigma16,
                        float* Rout, int64_t ldr, void* ws, hipStream_t st);


ptq_status pack_codes_launch(const uint8_t* codes, int64_t ldc, int64_t m, int64_t n, int bits, uint32_t* packed,
                             hipStream_t st);
ptq_status unpack_dequant_launch(const uint32_t* packed, int64_t m, int64_t n, int bits, const float* scales,
                                 const uint8_t* zeros, int group, double* Wq, int64_t ldq, hipStream_t st);
ptq_status pack_grids_launch(const float* scales, const uint8_t* zeros, int64_t m, int64_t ng, float* scales_t,
                             uint8_t* zeros_t, hipStream_t st);
size_t linear_forward_workspace_bytes(int64_t tokens, int64_t m, int64_t n, int64_t r);
// the per-GPU static scratch of ptq_lopro_linear_forward_static: its size, and its address on the current device
size_t linear_forward_static_scratch_bytes();
ptq_status linear_forward_static_scratch(void** ptr);
ptq_status linear_forward_launch(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m, int64_t n,
                                 const uint32_t* packed, int bits, const float* scales, const uint8_t* zeros,
                                 int group, const int32_t* perm, int b_I, int b_H, const uint8_t* U,
                                 const uint8_t* V, const uint16_t* sigma, int r, const double* s, float* O,
                                 int64_t ldo, void* ws, hipStream_t st);

}  // namespace ptq
