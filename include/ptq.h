/*
 * libptq -- layer-wise post-training weight quantization on one MI355X (gfx950).
 *
 * The library solves, for one linear layer with weight W (m x n, n = input
 * channels) and calibration input X (t tokens x n channels),
 *
 *        min_Q || W X^T - Q X^T ||_F        (paper Sec. 2, Eq. 1; Sec. 3.2, Eq. 8)
 *
 * by the column-sequential quantize-and-compensate scheme the paper uses as
 * its quantization step (Sec. 2, "Solution to O1" item (a); Algorithm 1,
 * stage C): accumulate the proxy Hessian H = X^T X, factor the damped inverse,
 * walk over the columns of W, and report the layer error.
 *
 * Conventions for every call
 *   - All matrices are row-major with an explicit leading dimension (in
 *     elements).  Every data pointer is a DEVICE pointer unless stated.
 *   - The caller owns every buffer, including the workspace whose size
 *     ptq_workspace_bytes() returns; the library allocates no device memory,
 *     keeps no data between calls and never frees anything.  (What it does keep,
 *     per device and for the life of the process: kernel attributes it has set,
 *     and two helper streams with a few events that ptq_damped_cholesky_inv
 *     creates on its first call for a wide factor (from about 5800 columns).)
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without waiting for it.
 *   - The return value reports errors the host can see (bad arguments, shapes,
 *     workspace too small, a failed launch).  Conditions only the device can
 *     see are written to a caller-provided device `info` array.
 *   - Workspaces must be 256-byte aligned.
 */
#ifndef PTQ_H
#define PTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PTQ_OK = 0,
  PTQ_ERR_ARG = 1,       /* null pointer, negative damp, bits outside [2,8]  */
  PTQ_ERR_SHAPE = 2,     /* sizes / leading dimensions / divisibility         */
  PTQ_ERR_DTYPE = 3,     /* storage type not supported by this call           */
  PTQ_ERR_WORKSPACE = 4, /* workspace missing, misaligned or too small        */
  PTQ_ERR_NOT_SPD = 5,   /* only ever written to `info`, never returned       */
  PTQ_ERR_HIP = 6        /* a HIP runtime call failed                         */
} ptq_status;

typedef enum { PTQ_F32 = 0, PTQ_BF16 = 1, PTQ_F64 = 2 } ptq_dtype;

typedef enum {
  PTQ_OP_HESSIAN = 0,
  PTQ_OP_CHOLESKY_INV = 1,
  PTQ_OP_QUANTIZE = 2,
  PTQ_OP_LAYER_ERROR = 3,
  PTQ_OP_LOPRO_ORDER = 4,
  PTQ_OP_LOPRO_ROTATE_HESSIAN = 5,
  PTQ_OP_ACTIVATION_ABS_SUM = 6,
  PTQ_OP_SCALED_R1SVD = 7,
  PTQ_OP_LINEAR_FORWARD = 8 /* t = tokens, block = rank r */
} ptq_op;

typedef void* ptq_stream; /* hipStream_t */

/* Static, NUL-terminated description of a status code. */
const char* ptq_status_string(ptq_status s);

/*
 * Bytes of device workspace the given call needs for these sizes
 * (m, t, block are ignored by ops that do not use them; pass 0).
 * `bytes` is a host pointer.
 */
ptq_status ptq_workspace_bytes(ptq_op op, int64_t m, int64_t n, int64_t t, int64_t block,
                               size_t* bytes);

/*
 * Proxy Hessian accumulation (Sec. 2, Eq. 1:  H = E[x x^T], taken as the raw
 * sum over tokens; Algorithm 1 computes it once per layer).
 *
 *   H[i][j] += sum_k X[k][i] * X[k][j]      for all 0 <= i <= j < n
 *
 * H    n x n float64, leading dimension ldh >= n.  Accumulated in place, so the
 *      caller zeroes it before the first chunk of tokens.  Only the upper
 *      triangle (i <= j) is defined on return; entries below the diagonal may
 *      be left untouched or overwritten with their mirror values.
 * X    t x n, tokens by channels, PTQ_BF16 (raw bfloat16 bits) or PTQ_F32,
 *      leading dimension ldx >= n.  Read only.  bf16 needs n % 8 == 0 and
 *      ldx % 8 == 0 and a 16-byte aligned X (vector loads); f32 has no such rule.
 * t may be 0 (no-op).  Products of bf16 inputs are exact; partial sums run in
 * float32 over at most 20480 tokens (65536 for layers wider than about 8000
 * channels) and are added to H in float64 in a fixed order.
 * Errors: PTQ_ERR_ARG (null), PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_hessian_accumulate(double* H, int64_t ldh, const void* X, ptq_dtype xdt, int64_t t,
                                  int64_t n, int64_t ldx, void* ws, size_t ws_bytes,
                                  ptq_stream stream);

/*
 * Damped Cholesky factor of the inverse Hessian -- the coefficients with
 * which a column's quantization error is pushed onto the later columns
 * (the paper delegates this step to its quantization tool, Algorithm 1 stage C;
 * the factor is the one of the damped inverse).
 *
 *   H'   = H with H_jj = 1 wherever H_jj == 0 (a channel that never fired)
 *   H_d  = H' + damp * mean_j(H'_jj) * I
 *   U    = the upper-triangular matrix with positive diagonal, U^T U = H_d^{-1}
 *
 * H          n x n float64, only its upper triangle is read.  Not modified.
 * U          n x n float64 output, ldu >= n; the strict lower triangle is zeroed.
 * dead_mask  n bytes output, may be NULL: 1 where H_jj == 0.
 * info       2 x int32 device output, required: {PTQ_OK, 0}, or
 *            {PTQ_ERR_NOT_SPD, j} when the pivot of column j (in the order of
 *            elimination, j counted in H's own indexing) was not positive;
 *            U is then undefined.
 * For the largest factors two parts of a node's work run on the library's two helper streams
 * beside the rest (forked from and joined back into `stream` with events, so to the caller the
 * call is ordered on `stream` like any other, also under stream capture); calls from several
 * host threads on one device are serialised on a lock while they enqueue.
 * Errors: PTQ_ERR_ARG (null, damp < 0 or not finite), PTQ_ERR_SHAPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_damped_cholesky_inv(const double* H, int64_t ldh, int64_t n, double damp, double* U,
                                   int64_t ldu, uint8_t* dead_mask, int32_t* info, void* ws,
                                   size_t ws_bytes, ptq_stream stream);

/*
 * Blocked column-by-column quantization with error compensation (Sec. 2,
 * item (a): columns are quantized one after another and each column's error
 * is compensated in the columns that follow).  For every row of W and
 * j = 0 .. n-1, with w the row's current (already compensated) values:
 *
 *   when j is the first column of a group of `group` columns:
 *       lo = min(0, min w[group]),  hi = max(0, max w[group]),
 *       (lo, hi) = (-1, 1) if lo == hi,
 *       scale = float32((hi - lo) / (2^bits - 1)),  zero = rne(-lo / scale)
 *   code_j = clamp(rne(w_j / scale) + zero, 0, 2^bits - 1)
 *   q_j    = scale * (code_j - zero)
 *   e_j    = (w_j - q_j) / U_jj
 *   w_k   -= e_j * U_jk            for all k > j
 *
 * (rne = round half to even).  The update of the columns outside the current
 * block of `block` columns is applied lazily, once per block; `block` changes
 * the order of summation only.
 *
 * W          m x n, PTQ_F32 / PTQ_BF16 / PTQ_F64, ldw >= n.  Not modified.
 * U          n x n float64 upper-triangular factor from ptq_damped_cholesky_inv.
 * dead_mask  n bytes or NULL; columns with mask 1 are treated as all-zero.
 * bits       2..8.   group > 0 with n % group == 0.
 * block      > 0, a multiple of 16, at most 256, and block % group == 0 or
 *            group % block == 0.  n need not be a multiple of block.
 * codes      m x n uint8 output, one code per byte, row-major, ld = n.
 * scales     m x (n/group) float32 output.   zeros  m x (n/group) uint8 output.
 * Wq         m x n float64 output with ld = n, or NULL: the dequantized weights.
 * row_err2   m float64 output or NULL: sum_j e_j^2 of each row.
 * Errors: PTQ_ERR_ARG, PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_quantize_layer(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                              const double* U, int64_t ldu, const uint8_t* dead_mask, int bits,
                              int group, int block, uint8_t* codes, float* scales, uint8_t* zeros,
                              double* Wq, double* row_err2, void* ws, size_t ws_bytes,
                              ptq_stream stream);

/*
 * The same solve with STATIC GROUPS, an option of the quantizer the paper builds on (Sec. 2,
 * item (a): compensation-based methods, GPTQ): the scale and zero of every (row, group) are
 * taken from W as it is handed over (dead columns counting as zeros), before any compensation,
 * instead of from the row's updated values when the walk reaches the group.  Arguments, layouts,
 * workspace and errors as for ptq_quantize_layer.  (Its other option, taking the columns in the
 * order of falling diag(H), needs no entry point: ptq_lopro_column_order on a 1 x n matrix of
 * ones gives that order, and the permutation calls with b_I = n apply it without rotating.)
 */
ptq_status ptq_quantize_layer_static_groups(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m,
                                            int64_t n, const double* U, int64_t ldu,
                                            const uint8_t* dead_mask, int bits, int group, int block,
                                            uint8_t* codes, float* scales, uint8_t* zeros, double* Wq,
                                            double* row_err2, void* ws, size_t ws_bytes,
                                            ptq_stream stream);

/*
 * The same solve with a VECTOR quantizer (the paper's second variant; implementation-details
 * appendix: a randomly drawn, untrained codebook, no block-wise scaling, vectors of 4 weights at
 * 2 bits per weight and of 2 weights at 3 bits per weight; assignment by the proxy-Hessian loss,
 * Sec. 3.2, Eq. 8; Algorithm 1, quantization step).  A vector is `dim` consecutive columns of a row
 * starting at a multiple of dim.  For every row and group g = columns [j, j + dim), j = g dim, with w
 * the row's current (compensated) values and T = U[j:j+dim, j:j+dim]:
 *
 *   loss(c)  = sum_i e_i^2,   e = (w - c) T^-1   (the errors of the group's columns, one after the other)
 *   index_g  = the entry of the codebook with the smallest loss (the lowest index among equal ones)
 *   w_k     -= sum_i e_i U[j+i][k]    for all later columns k
 *
 * codebook   entries x dim float32, row-major, in the weights' own units; one codebook for the layer,
 *            drawn by the caller.  1 <= entries <= 256; dim is 1, 2 or 4; n % dim == 0.
 * indices    m x (n / dim) uint8 output, row-major.
 * Wq         m x n float64 output (ld = n) or NULL: the assigned entries.   row_err2  m float64 or NULL.
 * W, U, dead_mask, block (a multiple of 16, at most 256), workspace (PTQ_OP_QUANTIZE) and errors as for
 * ptq_quantize_layer.  All arithmetic is float64.
 */
ptq_status ptq_quantize_layer_vq(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                                 const double* U, int64_t ldu, const uint8_t* dead_mask, const float* codebook,
                                 int entries, int dim, int block, uint8_t* indices, double* Wq,
                                 double* row_err2, void* ws, size_t ws_bytes, ptq_stream stream);

/*
 * Relative layer error under the proxy-Hessian loss (Sec. 2, Eq. 1):
 *
 *   num = tr((W - Wq) H (W - Wq)^T),  den = tr(W H W^T),  rel = sqrt(num / den)
 *
 * which equals ||W X^T - Wq X^T||_F / ||W X^T||_F for H = X^T X.  Pass the
 * undamped H; only its upper triangle is read.
 *
 * W   m x n, PTQ_F32 / PTQ_BF16 / PTQ_F64, ldw >= n.   Wq  m x n float64, ld = n.
 * out 3 x float64 device output: {rel, num, den}.
 * Precision follows the storage type of W.  PTQ_F64: float64 throughout.  PTQ_F32 / PTQ_BF16:
 * W - Wq, W and H are rounded to float32 once, their products are formed from bfloat16 pieces of
 * the float32 values, the sums over the inner index run in float32 on the matrix cores, and the
 * sums over the m x n entries are float64.  Layers of fewer than 65536 entries use three pieces
 * (products complete to 2^-24): num and den agree with the float64 definition to about 1e-8
 * relative (3e-7 at worst, for a layer of a single entry).  Larger layers use two pieces (products
 * complete to 2^-16, errors unbiased and averaged over the m x n terms): num and den agree to
 * about 1e-6 relative and rel to about 1e-7 (the agreement asked of rel is 1e-4).  Sums are taken
 * in a fixed order: results are reproducible.
 * Errors: PTQ_ERR_ARG, PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_layer_error(const void* W, ptq_dtype wdt, int64_t ldw, const double* Wq, int64_t m,
                           int64_t n, const double* H, int64_t ldh, double* out, void* ws,
                           size_t ws_bytes, ptq_stream stream);

/* ---------------------------------------------------------------------------
 * LoPRo's pre-conditioning of the same solve (Sec. 3.2): the residual R and the
 * proxy Hessian are taken to a permuted, partially rotated basis, the solve
 * above runs there unchanged on (R', H'), and its result is taken back.
 *
 *   perm  orders the columns by  diag(H) / amean(R, axis=0)            (Eq. 5)
 *   P     applies perm as a gather: column c of (R P) is column perm[c] of R
 *   Q     = blockdiag(I_{b_I}, H_wal, .., H_wal), H_wal the b_H x b_H Sylvester
 *         Hadamard matrix times 1/sqrt(b_H)                            (Eq. 6)
 *   R'    = R P Q        H' = Q^T P^T H P Q        W = W_r + Q(R') Q^T P^T   (Eq. 6-8)
 *
 * b_H is a power of two, 16 <= b_H <= 256; b_I >= 0 is a multiple of 4; (n - b_I) is a
 * multiple of b_H; n is a multiple of 4.  Violations: PTQ_ERR_SHAPE.
 * ------------------------------------------------------------------------- */

/*
 * Column order (Eq. 5).  key_j = H_jj / mean_i |R_ij|; a column whose residual is all zero
 * gets +inf if H_jj > 0 and 0 otherwise.  perm lists the columns by descending key
 * (descending != 0: the columns the paper calls important come first, which is what the
 * identity block of Q is for) or by ascending key (descending == 0: Eq. 5 read literally);
 * equal keys keep the lower column index first.
 *
 * R     m x n, PTQ_F32 / PTQ_BF16 / PTQ_F64, ldr >= n.    H   n x n float64, diagonal read.
 * perm  n int32 output.     keys  n float64 output or NULL.
 * Errors: PTQ_ERR_ARG, PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_lopro_column_order(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                  const double* H, int64_t ldh, int descending, int32_t* perm,
                                  double* keys, void* ws, size_t ws_bytes, ptq_stream stream);

/*
 * R' = R P Q (Eq. 6).   Rout  m x n float64, ldo >= n, 32-byte aligned rows (ldo % 4 == 0).
 * For bf16 / f32 inputs of moderate dynamic range and b_H = 16, 64 or 256 every sum is exact.
 * perm must be a permutation of 0..n-1 (not checked).  No workspace.
 */
ptq_status ptq_lopro_rotate_weight(const void* R, ptq_dtype rdt, int64_t ldr, int64_t m, int64_t n,
                                   const int32_t* perm, int b_I, int b_H, double* Rout, int64_t ldo,
                                   ptq_stream stream);

/*
 * Wout = Rq Q^T P^T (Eq. 7): a matrix given in the rotated basis, e.g. the dequantized
 * result of the solve, back in the layer's own column order.  Rq, Wout m x n float64;
 * Rq needs ldq % 4 == 0 and a 32-byte aligned base.  Wout must not alias Rq.
 */
ptq_status ptq_lopro_unrotate_weight(const double* Rq, int64_t ldq, int64_t m, int64_t n,
                                     const int32_t* perm, int b_I, int b_H, double* Wout, int64_t ldo,
                                     ptq_stream stream);

/*
 * H' = Q^T P^T H P Q (Eq. 8).  Only the upper triangle of H is read; Hout (n x n float64,
 * ldo >= n, ldo % 4 == 0, must not alias H) receives the full symmetric matrix.
 */
ptq_status ptq_lopro_rotate_hessian(const double* H, int64_t ldh, int64_t n, const int32_t* perm,
                                    int b_I, int b_H, double* Hout, int64_t ldo, void* ws,
                                    size_t ws_bytes, ptq_stream stream);

/* ---------------------------------------------------------------------------
 * The low-rank step that produces the residual R (Sec. 3.1, Eq. 4: W = W_r + R with
 * W_r from a decomposition of the activation-scaled weight; Sec. 3.3: the rank-one
 * randomized sketch "R1SVD"; Algorithm 1, the lines before the permutation).
 * ------------------------------------------------------------------------- */

/*
 * Per-channel activation magnitude (Algorithm 1: Xbar = mean(|X|, axis 0)), kept as a raw
 * sum so that calibration batches can be streamed:
 *
 *   asum[j] += sum_k |X[k][j]|
 *
 * asum  n float64, accumulated in place (zero it before the first batch).
 * X     t x n, PTQ_F32 or PTQ_BF16, ldx >= n; n and ldx multiples of 8, base 16-byte aligned.
 * Sums are float64 and taken in a fixed order.  Workspace: PTQ_OP_ACTIVATION_ABS_SUM.
 * Errors: PTQ_ERR_ARG, PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE.
 */
ptq_status ptq_activation_abs_sum(double* asum, const void* X, ptq_dtype xdt, int64_t t, int64_t n,
                                  int64_t ldx, void* ws, size_t ws_bytes, ptq_stream stream);

/*
 * The scale of Algorithm 1 from the accumulated sums:  Xbar = asum / tokens,
 *   s_j = Xbar_j^2.5 / sqrt(max(Xbar) * min(Xbar)).
 * max and min run over the channels with Xbar_j > 0; a channel that was never active gets
 * s_j = 1 (the printed formula has no value there).   s  n float64 output.  No workspace.
 */
ptq_status ptq_activation_scale(const double* asum, int64_t tokens, int64_t n, double* s,
                                ptq_stream stream);

/*
 * Scaled rank-one sketching (Sec. 3.3, Eq. 9-11; Algorithm 1).  With A = W diag(s), for
 * k = 0 .. r-1:
 *     y = (A A^T)^it A S[k],   p = A^T y,
 *     U[k] = e4m3(y / ||y||),  V[k] = e4m3(p / ||p||),  sigma[k] = fp16(||p|| / ||y||),
 *     A <- A - sigma[k] U[k] V[k]^T      (with the stored, rounded values)
 * and finally  R = A diag(s)^-1, so that  W = (U^T diag(sigma) V) diag(s)^-1 + R  holds for
 * what is stored.  If y or p is zero the rank stores zeros.
 *
 * W      m x n, PTQ_F32 / PTQ_BF16 / PTQ_F64, ldw >= n.      s  n float64, all entries nonzero.
 * S      r x n float32 with leading dimension lds >= n, lds % 4 == 0, 16-byte aligned: the
 *        random vector of each rank (the caller draws them; standard normal in the paper's
 *        prototype).
 * U, V   r x m and r x n bytes, dense: OCP e4m3 codes (bias 7, no infinities), conversion
 *        rounds to nearest, ties to even.      sigma  r IEEE binary16 bit patterns; a value
 *        beyond the format's range is stored as 65504 (the deflation then removes part of
 *        that direction and later ranks find the rest).
 * R      m x n float32 output, ldr >= n, ldr % 4 == 0, 16-byte aligned.  May not alias W.
 * r, it  rank and number of power iterations (the paper uses 16 and 8); r = 0 gives R = W.
 * n % 4 == 0 and n <= 32768.
 * The running matrix W diag(s) - sum of the stored rank-one terms is held in float32 and
 * rewritten at every rank, or -- for a bfloat16 W with n % 8 == 0, ldw % 8 == 0, 16-byte aligned,
 * r <= 16, too large for the first case -- never formed: the products are taken from W as it
 * is (kept on the chip if it fits there, else streamed) and the stored ranks are applied as
 * corrections.  Sums across threads are float64 in a fixed order: results are reproducible
 * run to run.
 * The loop runs as ONE cooperative launch where the device can hold it, its workgroups waiting
 * for each other's partial sums; a workgroup that waits longer than a fixed number of rounds
 * (about a second) gives up and makes all others give up: the call still completes, and every
 * entry of sigma is then the NaN pattern 0x7e00 (check sigma[0] after synchronising).
 * Workspace: PTQ_OP_SCALED_R1SVD (m, n).
 * Errors: PTQ_ERR_ARG, PTQ_ERR_SHAPE, PTQ_ERR_DTYPE, PTQ_ERR_WORKSPACE, PTQ_ERR_HIP.
 */
ptq_status ptq_scaled_r1svd(const void* W, ptq_dtype wdt, int64_t ldw, int64_t m, int64_t n,
                            const double* s, const float* S, int64_t lds, int r, int it, uint8_t* U,
                            uint8_t* V, uint16_t* sigma, float* R, int64_t ldr, void* ws,
                            size_t ws_bytes, ptq_stream stream);

/* ---------------------------------------------------------------------------
 * What is stored for a layer and the form it is applied in (Algorithm 1, last lines: the
 * quantized residual, U, Sigma, V, the scale vector and the permutation; Sec. 3.4, Eq. 12:
 * its size; Sec. 3.2, Eq. 7 and the time-complexity appendix: its use).
 * ------------------------------------------------------------------------- */

/*
 * Eq. 12, host arithmetic only: average bits per weight of an m x n layer quantized to d_q
 * bits with one d_o-bit scale per group of g columns, rank-r factors in d_r bits, the scale
 * vector, the permutation and Sigma:
 *   d_q + d_o/g + r d_r/n + r d_r/m + 2 d_o/n + r d_o/(m n).     Returns -1 on bad arguments.
 */
double ptq_average_bits(int64_t m, int64_t n, double d_q, double d_o, int64_t g, int64_t r, double d_r);

/*
 * Bit packing.  32 consecutive codes of a row (a chunk) form a little-endian bit stream of
 * exactly `bits` 32-bit words, code j of the chunk in bits [j bits, (j+1) bits); chunks are
 * stored chunk-major: packed is (n / 32) x m x bits words (consecutive rows of a chunk are
 * adjacent, which is the order the forward kernel reads them in); 16-byte aligned.
 * codes m x n bytes (values < 2^bits; higher bits are ignored), ldc >= n, ldc % 16 == 0,
 * 16-byte aligned.  bits in {2, 3, 4, 8}; n % 32 == 0.
 * The grids are brought into the matching group-major order on the way: scales, zeros
 * (m x n/group, as ptq_quantize_layer wrote them) -> scales_t, zeros_t (n/group x m); pass
 * NULL for all four to pack the codes only.
 */
ptq_status ptq_pack_codes(const uint8_t* codes, int64_t ldc, int64_t m, int64_t n, int bits,
                          uint32_t* packed, const float* scales, const uint8_t* zeros, int group,
                          float* scales_t, uint8_t* zeros_t, ptq_stream stream);

/*
 * The inverse with dequantization:  Wq[i][j] = scale_t[j/group][i] * (code[i][j] - zero_t[j/group][i])
 * in float64 (exact: a float32 times a small integer), the value ptq_quantize_layer wrote.
 * scales_t n/group x m float32, zeros_t n/group x m bytes, Wq m x n float64, ldq >= n.
 */
ptq_status ptq_unpack_dequantize(const uint32_t* packed, int64_t m, int64_t n, int bits,
                                 const float* scales_t, const uint8_t* zeros_t, int group, double* Wq,
                                 int64_t ldq, ptq_stream stream);

/*
 * The stored layer applied to a few tokens (Eq. 7, rows = tokens):
 *     X~ = X P Q,      O = X~ Dequant(packed)^T + ((X diag(s)^-1) V^T diag(sigma)) U.
 * The residual stays in the rotated basis it was quantized in; the input is permuted and
 * rotated once (same perm, b_I, b_H and their restrictions as the rotation calls above).
 *
 * X      tokens x n, PTQ_F32 / PTQ_BF16 / PTQ_F64, ldx >= n.       O  tokens x m float32, ldo >= m.
 * packed, scales_t, zeros_t (group-major), bits, group: as above; group % 32 == 0.
 * U, V   r x m and r x n e4m3 codes, sigma r fp16 bit patterns, s n float64: the output of
 *        ptq_scaled_r1svd; r = 0 applies the residual alone (U, V, sigma, s may be NULL).
 * X~ and the low-rank coefficients are formed in float64 and rounded to float32; the products
 * with the codes accumulate in float32.  tokens <= 4096 (meant for a handful: the call reads
 * the packed codes once per pass, and a pass takes up to 32 tokens when there are eight or
 * more of them, up to four otherwise).
 * Workspace: PTQ_OP_LINEAR_FORWARD with m, n, t = tokens and block = r.
 */
ptq_status ptq_lopro_linear_forward(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m,
                                    int64_t n, const uint32_t* packed, int bits, const float* scales_t,
                                    const uint8_t* zeros_t, int group, const int32_t* perm, int b_I,
                                    int b_H, const uint8_t* U, const uint8_t* V, const uint16_t* sigma,
                                    int r, const double* s, float* O, int64_t ldo, void* ws,
                                    size_t ws_bytes, ptq_stream stream);

/*
 * ptq_lopro_linear_forward for callers that cannot allocate device memory or pass a workspace
 * along: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as ptq_lopro_linear_forward, without the workspace: the
 * scratch memory (rotated input, low-rank coefficients, partial sums, row-block counters) is a
 * fixed array of ptq_lopro_linear_forward_static_limit() bytes (32 MiB) that is part of the
 * library's device code, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing.  A problem whose PTQ_OP_LINEAR_FORWARD workspace size exceeds the limit is
 * refused with PTQ_ERR_WORKSPACE (the limit covers, e.g., 11008 x 4096 and 4096 x 11008 layers
 * with up to 64 tokens).  All calls on one GPU share that GPU's array: calls that overlap on one
 * GPU (different streams, or different host threads) race and must be serialised by the caller;
 * calls on different GPUs are independent.  What has to start at zero is cleared by the call's
 * own kernels on `stream`.
 */
size_t ptq_lopro_linear_forward_static_limit(void);
ptq_status ptq_lopro_linear_forward_static(const void* X, ptq_dtype xdt, int64_t ldx, int64_t tokens, int64_t m,
                                           int64_t n, const uint32_t* packed, int bits, const float* scales_t,
                                           const uint8_t* zeros_t, int group, const int32_t* perm, int b_I,
                                           int b_H, const uint8_t* U, const uint8_t* V, const uint16_t* sigma,
                                           int r, const double* s, float* O, int64_t ldo, ptq_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* PTQ_H */
