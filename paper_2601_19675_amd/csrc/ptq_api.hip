// C ABI of libptq: argument checks, then the per-step launchers.
#include "common.h"

#include <cmath>

using namespace ptq;

namespace {
bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }
bool ws_bad(const void* ws, size_t have, size_t need) {
  return need > 0 && (ws == nullptr || misaligned(ws, 256) || have < need);
}
bool dtype_ok(ptq_dtype d) { return d == PTQ_F32 || d == PTQ_BF16 || d == PTQ_F64; }
// shape rules shared by the rotation calls
bool rotation_shape_bad(int64_t n, int b_I, int b_H) {
  if (b_H < 16 || b_H > 256 || (b_H & (b_H - 1)) != 0) return true;
  if (b_I < 0 || b_I > n || b_I % 4 != 0 || n % 4 != 0) return true;
  return (n - b_I) % b_H != 0;
}
}  // namespace

extern "C" {

const char* ptq_status_string(ptq_status s) {
  switch (s) {
    case PTQ_OK: return "ok";
    case PTQ_ERR_ARG: return "invalid argument";
    case PTQ_ERR_SHAPE: return "invalid shape or leading dimension";
    case PTQ_ERR_DTYPE: return "unsupported storage type";
    case PTQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case PTQ_ERR_NOT_SPD: return "matrix not positive definite";
    case PTQ_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

ptq_status ptq_workspace_bytes(ptq_op op, int64_t m, int64_t n, int64_t t, int64_t block, size_t* bytes) {
  if (!bytes) return PTQ_ERR_ARG;
  if (m < 0 || n < 0 || t < 0) return PTQ_ERR_SHAPE;
  switch (op) {
    case PTQ_OP_HESSIAN: *bytes = hessian_workspace_bytes(n, t); return PTQ_OK;
    case PTQ_OP_CHOLESKY_INV: *bytes = cholesky_workspace_bytes(n); return PTQ_OK;
    case PTQ_OP_QUANTIZE: *bytes = quantize_workspace_bytes(m, n); return PTQ_OK;
    case PTQ_OP_LAYER_ERROR: *bytes = layer_error_workspace_bytes(m, n); return PTQ_OK;
    case PTQ_OP_LOPRO_ORDER: *bytes = lopro_order_workspace_bytes(n); return PTQ_OK;
    case PTQ_OP_LOPRO_ROTATE_HESSIAN: *bytes = lopro_hessian_workspace_bytes(n); return PTQ_OK;
    case PTQ_OP_ACTIVATION_ABS_SUM: *bytes = abs_sum_workspace_bytes(n); return PTQ_OK;
    case PTQ_OP_SCALED_R1SVD: *bytes = r1svd_workspace_bytes(m, n); return PTQ_OK;
    case PTQ_OP_LINEAR_FORWARD: *bytes = linear_forward_workspace_bytes(t, m, n, block); return PTQ_OK;
  }
  return PTQ_ERR_ARG;
}

ptq_status ptq_hessian_accumulate(double* H, int64_t ldh, const void* X, ptq_dtype xdt, int64_t t,
                                  int64_t n, int64_t ldx, void* ws, size_t ws_bytes, ptq_stream stream) {
  if (t < 0 || n < 0 || ldh < n || ldx < n || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (xdt != PTQ_F32 && xdt != PTQ_BF16) return PTQ_ERR_DTYPE;
  if (t == 0 || n == 0) return PTQ_OK;
  if (!H || !X) return PTQ_ERR_ARG;
  if (xdt == PTQ_BF16) {
    if (n % 8 != 0 || ldx % 8 != 0) return PTQ_ERR_SHAPE;
    if (misaligned(X, 16)) return PTQ_ERR_ARG;
  }
  if (ws_bad(ws, ws_bytes, hessian_workspace_bytes(n, t))) return PTQ_ERR_WORKSPACE;
  return hessian_launch(H, ldh, X, xdt, t, n, ldx, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

ptq_status ptq_damped_cholesky_inv(const double* H, int64_t ldh, int64_t n, double damp, double* U,
                                   int64_t ldu, uint8_t* dead_mask, int32_t* info, void* ws,
                                   size_t ws_bytes, ptq_stream stream) {
  if (n < 0 || ldh < n || ldu < n || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (!(damp >= 0.0) || !std::isfinite(damp)) return PTQ_ERR_ARG;
  if (n == 0) return PTQ_OK;
  if (!H || !U || !info) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, cholesky_workspace_bytes(n))) return PTQ_ERR_WORKSPACE;
  return cholesky_launch(H, ldh, n, damp, U, ldu, dead_mask, info, ws, ws_bytes,
                         static_cast<hipStream_t>(stream));
}

static ptq_status quantize_checked(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* U,
                                   int64_t ldu, const uint8_t* dead_mask, int bits, int group, int block,
                                   uint8_t* codes, float* scales, uint8_t* zeros, double* Wq, double* row_err2,
                                   int static_groups, void* ws, size_t ws_bytes, ptq_stream stream) {
  if (bits < 2 || bits > 8) return PTQ_ERR_ARG;
  if (!dtype_ok(wdt)) return PTQ_ERR_DTYPE;
  if (m < 0 || n < 0 || ldw < n || ldu < n || m > INT32_MAX / 2 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (group <= 0 || block <= 0 || n % group != 0) return PTQ_ERR_SHAPE;
  if (block % 16 != 0 || block > 256) return PTQ_ERR_SHAPE;
  if (block % group != 0 && group % block != 0) return PTQ_ERR_SHAPE;
  // groups start on 16-column mini-block boundaries and must fit one block
  if (group % 16 != 0 || group > 256) return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!W || !U || !codes || !scales || !zeros) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, quantize_workspace_bytes(m, n))) return PTQ_ERR_WORKSPACE;
  return quantize_launch(W, wdt, ldw, m, n, U, ldu, dead_mask, bits, group, block, codes, scales, zeros,
                         Wq, row_err2, static_groups, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

ptq_status ptq_quantize_layer(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                              const double* U, int64_t ldu, const uint8_t* dead_mask, int bits, int group,
                              int block, uint8_t* codes, float* scales, uint8_t* zeros, double* Wq,
                              double* row_err2, void* ws, size_t ws_bytes, ptq_stream stream) {
  return quantize_checked(W, wdt, ldw, m, n, U, ldu, dead_mask, bits, group, block, codes, scales, zeros, Wq,
                          row_err2, 0, ws, ws_bytes, stream);
}

ptq_status ptq_quantize_layer_static_groups(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                                            const double* U, int64_t ldu, const uint8_t* dead_mask, int bits,
                                            int group, int block, uint8_t* codes, float* scales, uint8_t* zeros,
                                            double* Wq, double* row_err2, void* ws, size_t ws_bytes,
                                            ptq_stream stream) {
  return quantize_checked(W, wdt, ldw, m, n, U, ldu, dead_mask, bits, group, block, codes, scales, zeros, Wq,
                          row_err2, 1, ws, ws_bytes, stream);
}

ptq_status ptq_quantize_layer_vq(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* U,
                                 int64_t ldu, const uint8_t* dead_mask, const float* codebook, int entries, int dim,
                                 int block, uint8_t* indices, double* Wq, double* row_err2, void* ws,
                                 size_t ws_bytes, ptq_stream stream) {
  if (entries < 1 || entries > 256 || (dim != 1 && dim != 2 && dim != 4)) return PTQ_ERR_ARG;
  if (!dtype_ok(wdt)) return PTQ_ERR_DTYPE;
  if (m < 0 || n < 0 || ldw < n || ldu < n || m > INT32_MAX / 2 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (n % dim != 0 || block <= 0 || block % 16 != 0 || block > 256) return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!W || !U || !codebook || !indices) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, quantize_workspace_bytes(m, n))) return PTQ_ERR_WORKSPACE;
  return quantize_vq_launch(W, wdt, ldw, m, n, U, ldu, dead_mask, codebook, entries, dim, block, indices, Wq,
                            row_err2, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

ptq_status ptq_layer_error(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                           int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                           size_t ws_bytes, ptq_stream stream) {
  if (!dtype_ok(wdt)) return PTQ_ERR_DTYPE;
  if (m <= 0 || n <= 0 || ldw < n || ldh < n || m > INT32_MAX / 2 || n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  if (!W || !Wq || !H || !out) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, layer_error_workspace_bytes(m, n))) return PTQ_ERR_WORKSPACE;
  return layer_error_launch(W, wdt, ldw, Wq, m, n, H, ldh, out, ws, ws_bytes,
                            static_cast<hipStream_t>(stream));
}

ptq_status ptq_lopro_column_order(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                  const double* H, int64_t ldh, int descending, int32_t* perm, double* keys,
                                  void* ws, size_t ws_bytes, ptq_stream stream) {
  if (!dtype_ok(rdt)) return PTQ_ERR_DTYPE;
  if (m <= 0 || n < 0 || ldr < n || ldh < n || m > INT32_MAX / 2 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (n == 0) return PTQ_OK;
  if (!R || !H || !perm) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, lopro_order_workspace_bytes(n))) return PTQ_ERR_WORKSPACE;
  return lopro_order_launch(R, rdt, ldr, m, n, H, ldh, descending, perm, keys, ws,
                            static_cast<hipStream_t>(stream));
}

ptq_status ptq_lopro_rotate_weight(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                   const int32_t* perm, int b_I, int b_H, double* Rout, int64_t ldo,
                                   ptq_stream stream) {
  if (!dtype_ok(rdt)) return PTQ_ERR_DTYPE;
  if (m < 0 || n < 0 || ldr < n || ldo < n || ldo % 4 != 0 || m > INT32_MAX / 2 || n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  if (rotation_shape_bad(n, b_I, b_H)) return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!R || !perm || !Rout || misaligned(Rout, 32) || misaligned(perm, 16)) return PTQ_ERR_ARG;
  return lopro_rotate_weight_launch(R, rdt, ldr, m, n, perm, b_I, b_H, Rout, ldo,
                                    static_cast<hipStream_t>(stream));
}

ptq_status ptq_lopro_unrotate_weight(const double* Rq, int64_t ldq, int64_t m, int64_t n, const int32_t* perm,
                                     int b_I, int b_H, double* Wout, int64_t ldo, ptq_stream stream) {
  if (m < 0 || n < 0 || ldq < n || ldq % 4 != 0 || ldo < n || m > INT32_MAX / 2 || n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  if (rotation_shape_bad(n, b_I, b_H)) return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!Rq || !perm || !Wout || Rq == Wout || misaligned(Rq, 32) || misaligned(perm, 16)) return PTQ_ERR_ARG;
  return lopro_unrotate_weight_launch(Rq, ldq, m, n, perm, b_I, b_H, Wout, ldo,
                                      static_cast<hipStream_t>(stream));
}

ptq_status ptq_lopro_rotate_hessian(const double* H, int64_t ldh, int64_t n, const int32_t* perm, int b_I,
                                    int b_H, double* Hout, int64_t ldo, void* ws, size_t ws_bytes,
                                    ptq_stream stream) {
  if (n < 0 || ldh < n || ldo < n || ldo % 4 != 0 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (rotation_shape_bad(n, b_I, b_H)) return PTQ_ERR_SHAPE;
  if (n == 0) return PTQ_OK;
  if (!H || !perm || !Hout || H == Hout || misaligned(Hout, 32) || misaligned(perm, 16)) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, lopro_hessian_workspace_bytes(n))) return PTQ_ERR_WORKSPACE;
  return lopro_rotate_hessian_launch(H, ldh, n, perm, b_I, b_H, Hout, ldo, ws,
                                     static_cast<hipStream_t>(stream));
}

ptq_status ptq_activation_abs_sum(double* asum, const void* X, ptq_dtype xdt, int64_t t, int64_t n, int64_t ldx,
                                  void* ws, size_t ws_bytes, ptq_stream stream) {
  if (xdt != PTQ_F32 && xdt != PTQ_BF16) return PTQ_ERR_DTYPE;
  if (t < 0 || n < 0 || ldx < n || n % 8 != 0 || ldx % 8 != 0 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (t == 0 || n == 0) return PTQ_OK;
  if (!asum || !X || misaligned(X, 16)) return PTQ_ERR_ARG;
  if (ws_bad(ws, ws_bytes, abs_sum_workspace_bytes(n))) return PTQ_ERR_WORKSPACE;
  return abs_sum_launch(asum, X, xdt, t, n, ldx, ws, static_cast<hipStream_t>(stream));
}

ptq_status ptq_activation_scale(const double* asum, int64_t tokens, int64_t n, double* s, ptq_stream stream) {
  if (tokens <= 0 || n < 0 || n > INT32_MAX / 2) return PTQ_ERR_SHAPE;
  if (n == 0) return PTQ_OK;
  if (!asum || !s) return PTQ_ERR_ARG;
  return activation_scale_launch(asum, tokens, n, s, static_cast<hipStream_t>(stream));
}

ptq_status ptq_scaled_r1svd(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n, const double* s,
                            const float* S, int64_t lds, int r, int it, uint8_t* U, uint8_t* V,
                            uint16_t* sigma, float* R, int64_t ldr, void* ws, size_t ws_bytes,
                            ptq_stream stream) {
  if (!dtype_ok(wdt)) return PTQ_ERR_DTYPE;
  if (m <= 0 || n <= 0 || ldw < n || ldr < n || ldr % 4 != 0 || n % 4 != 0 || lds < n || m > INT32_MAX / 2 ||
      n > r1svd_max_columns())
    return PTQ_ERR_SHAPE;
  if (r < 0 || r > 1024 || it < 0 || it > 1024) return PTQ_ERR_ARG;
  if (!W || !s || !R || misaligned(R, 16) || static_cast<const void*>(R) == W) return PTQ_ERR_ARG;
  if (r > 0 && (!S || !U || !V || !sigma || misaligned(S, 16))) return PTQ_ERR_ARG;
  if (lds % 4 != 0) return PTQ_ERR_SHAPE;
  if (ws_bad(ws, ws_bytes, r1svd_workspace_bytes(m, n))) return PTQ_ERR_WORKSPACE;
  return r1svd_launch(W, wdt, ldw, m, n, s, S, lds, r, it, U, V, sigma, R, ldr, ws,
                      static_cast<hipStream_t>(stream));
}

// For the library's own tests: selects the launch form of ptq_scaled_r1svd (0 = by shape, 1 = resident,
// 2 = stream, 3 = row blocks, 4 = one launch per step) and the spin limit of its bounded waits
// (negative = default) for all later calls of this process.  Deliberately not declared in ptq.h.
void ptq_internal_r1svd_select(int launch_form, long long spin_limit) { r1svd_select(launch_form, spin_limit); }

double ptq_average_bits(int64_t m, int64_t n, double d_q, double d_o, int64_t g, int64_t r, double d_r) {
  if (m <= 0 || n <= 0 || g <= 0 || r < 0) return -1.0;
  return d_q + d_o / (double)g + (double)r * d_r / (double)n + (double)r * d_r / (double)m + 2.0 * d_o / (double)n +
         (double)r * d_o / ((double)m * (double)n);
}

ptq_status ptq_pack_codes(const uint8_t* codes, int64_t ldc, int64_t m, int64_t n, int bits, uint32_t* packed,
                          const float* scales, const uint8_t* zeros, int group, float* scales_t, uint8_t* zeros_t,
                          ptq_stream stream) {
  if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return PTQ_ERR_ARG;
  if (m < 0 || n < 0 || n % 32 != 0 || ldc < n || ldc % 16 != 0 || m > INT32_MAX / 2 || n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  const bool grids = scales || zeros || scales_t || zeros_t;
  if (grids && (group <= 0 || n % group != 0)) return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!codes || !packed || misaligned(codes, 16) || misaligned(packed, 16)) return PTQ_ERR_ARG;
  if (grids && (!scales || !zeros || !scales_t || !zeros_t || scales == scales_t || zeros == zeros_t))
    return PTQ_ERR_ARG;
  ptq_status rc = pack_codes_launch(codes, ldc, m, n, bits, packed, static_cast<hipStream_t>(stream));
  if (rc != PTQ_OK || !grids) return rc;
  return pack_grids_launch(scales, zeros, m, n / group, scales_t, zeros_t, static_cast<hipStream_t>(stream));
}

ptq_status ptq_unpack_dequantize(const uint32_t* packed, int64_t m, int64_t n, int bits, const float* scales,
                                 const uint8_t* zeros, int group, double* Wq, int64_t ldq, ptq_stream stream) {
  if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return PTQ_ERR_ARG;
  if (m < 0 || n < 0 || n % 32 != 0 || group <= 0 || n % group != 0 || ldq < n || m > INT32_MAX / 2 ||
      n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  if (m == 0 || n == 0) return PTQ_OK;
  if (!packed || !scales || !zeros || !Wq || misaligned(packed, 16)) return PTQ_ERR_ARG;
  return unpack_dequant_launch(packed, m, n, bits, scales, zeros, group, Wq, ldq, static_cast<hipStream_t>(stream));
}

static ptq_status linear_forward_args(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m, int64_t n,
                                      const uint32_t* packed, int bits, const float* scales, const uint8_t* zeros,
                                      int group, const int32_t* perm, int b_I, int b_H, const uint8_t* U,
                                      const uint8_t* V, const uint16_t* sigma, int r, const double* s, float* O,
                                      int64_t ldo) {
  if (!dtype_ok(xdt)) return PTQ_ERR_DTYPE;
  if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return PTQ_ERR_ARG;
  if (tokens < 0 || tokens > 4096 || m <= 0 || n <= 0 || n % 32 != 0 || group <= 0 || group % 32 != 0 ||
      n % group != 0 || ldx < n || ldo < m || m > INT32_MAX / 2 || n > INT32_MAX / 2)
    return PTQ_ERR_SHAPE;
  if (rotation_shape_bad(n, b_I, b_H)) return PTQ_ERR_SHAPE;
  if (r < 0 || r > 1024) return PTQ_ERR_ARG;
  if (tokens == 0) return PTQ_OK;
  if (!X || !packed || !scales || !zeros || !perm || !O || misaligned(perm, 16) || misaligned(packed, 16))
    return PTQ_ERR_ARG;
  if (r > 0 && (!U || !V || !sigma || !s)) return PTQ_ERR_ARG;
  return PTQ_OK;
}

ptq_status ptq_lopro_linear_forward(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m, int64_t n,
                                    const uint32_t* packed, int bits, const float* scales, const uint8_t* zeros,
                                    int group, const int32_t* perm, int b_I, int b_H, const uint8_t* U,
                                    const uint8_t* V, const uint16_t* sigma, int r, const double* s, float* O,
                                    int64_t ldo, void* ws, size_t ws_bytes, ptq_stream stream) {
  const ptq_status rc = linear_forward_args(X, xdt, ldx, tokens, m, n, packed, bits, scales, zeros, group, perm, b_I,
                                            b_H, U, V, sigma, r, s, O, ldo);
  if (rc != PTQ_OK || tokens == 0) return rc;
  if (ws_bad(ws, ws_bytes, linear_forward_workspace_bytes(tokens, m, n, r))) return PTQ_ERR_WORKSPACE;
  return linear_forward_launch(X, xdt, ldx, tokens, m, n, packed, bits, scales, zeros, group, perm, b_I, b_H, U, V,
                               sigma, r, s, O, ldo, ws, static_cast<hipStream_t>(stream));
}

size_t ptq_lopro_linear_forward_static_limit(void) { return linear_forward_static_scratch_bytes(); }

ptq_status ptq_lopro_linear_forward_static(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m,
                                           int64_t n, const uint32_t* packed, int bits, const float* scales,
                                           const uint8_t* zeros, int group, const int32_t* perm, int b_I, int b_H,
                                           const uint8_t* U, const uint8_t* V, const uint16_t* sigma, int r,
                                           const double* s, float* O, int64_t ldo, ptq_stream stream) {
  const ptq_status rc = linear_forward_args(X, xdt, ldx, tokens, m, n, packed, bits, scales, zeros, group, perm, b_I,
                                            b_H, U, V, sigma, r, s, O, ldo);
  if (rc != PTQ_OK || tokens == 0) return rc;
  // sizes beyond the static array are refused, never trimmed
  if (linear_forward_workspace_bytes(tokens, m, n, r) > linear_forward_static_scratch_bytes()) return PTQ_ERR_WORKSPACE;
  void* ws = nullptr;
  const ptq_status sc = linear_forward_static_scratch(&ws);
  if (sc != PTQ_OK) return sc;
  return linear_forward_launch(X, xdt, ldx, tokens, m, n, packed, bits, scales, zeros, group, perm, b_I, b_H, U, V,
                               sigma, r, s, O, ldo, ws, static_cast<hipStream_t>(stream));
}

}  // extern "C"
