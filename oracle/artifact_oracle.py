"""CPU oracle for what LoPRo stores per layer and for the form inference uses it in.

TEST INFRASTRUCTURE ONLY (see ptq_oracle.py): plain numpy, float64, dense matrices.  Nothing
here is imported by the product path and no code is shared with the HIP kernels.

What the paper fixes (LoPRo, arXiv 2601.19675):
  * what is saved for a layer (Algorithm 1, last lines; stage C of its walk-through): the
    quantized residual W_q, the factors U, Sigma, V, the scale vector and the permutation;
  * how many bits per weight that is (Sec. 3.4, Eq. 12 and the average-bit appendix):
        d_C = d_q + d_o/g + r d_r/n + r d_r/m + 2 d_o/n + r d_o/(m n);
  * the form the layer is applied in (Sec. 3.2, Eq. 7; the time-complexity appendix): the
    input is permuted and rotated once, X~ = Q^T P^T X, the quantized residual multiplies X~,
    and the low-rank part is two thin products,  O = Dequant(W_q) X~ + U (Sigma (V' X)),
    V' = V diag(s)^-1 (Eq. 3).

Readings:
  * Bit packing is not specified: 32 consecutive codes of a row (a chunk) form a little-endian
    bit stream of exactly d_q 32-bit words, code j in bits [j d_q, (j+1) d_q); chunks are stored
    chunk-major, packed[chunk, row, word].  Any packing has the same size; this one is what the
    GPU kernels read (consecutive rows of a chunk are adjacent in memory).
  * Activations are handled as tokens x channels (rows are tokens), so X~ = X P Q and
    O = X~ Dequant(W_q)^T + ((X diag(s)^-1) V^T diag(sigma)) U.
  * Eq. 12 counts one d_o-bit scale per group and nothing for the zero-point of an
    asymmetric grid; `average_bits` is the printed formula, `stored_bits` counts what this
    build really stores (float32 scale and 8-bit zero-point per group, int32 permutation,
    float64 scale vector).

Parity status (tests/test_artifact_oracle_pins.py): Eq. 12 against the numbers the paper
prints for LLaMA-2 7B and 13B shapes (0.05 / 0.04 bits of low-rank overhead, 2.17 / 3.17 bits
in the result tables); packing against hand-worked words and the round trip; the inference
form against the dense definition  X (W_r + Q(R') Q^T P^T)^T  built from the other oracles.
"""
from __future__ import annotations

import numpy as np

from . import lopro_oracle as lo
from . import r1svd_oracle as ro


def average_bits(m: int, n: int, d_q: float, d_o: float, g: int, r: int, d_r: float,
                 terms: int = 6) -> float:
    """Eq. 12; `terms` < 6 drops trailing terms (the paper calls the last ones negligible)."""
    t = [d_q, d_o / g, r * d_r / n, r * d_r / m, 2.0 * d_o / n, r * d_o / (m * n)]
    return float(sum(t[:terms]))


def model_average_bits(shapes, d_q, d_o, g, r, d_r, terms: int = 6) -> float:
    """Parameter-weighted mean of Eq. 12 over the linear layers [(m, n), ...] of a model."""
    tot = sum(m * n for m, n in shapes)
    return float(sum(m * n * average_bits(m, n, d_q, d_o, g, r, d_r, terms) for m, n in shapes) / tot)


def stored_bits(m: int, n: int, d_q: int, g: int, r: int) -> float:
    """Bits per weight of what this build stores for a layer."""
    words = -(-n * d_q // 32)
    total = m * words * 32 + (m * n // g) * (32 + 8) + r * (m + n) * 8 + r * 16 + n * 32 + n * 64
    return total / (m * n)


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """uint8 codes (m x n, n % 32 == 0) -> uint32 words (n/32 x m x bits)."""
    m, n = codes.shape
    assert n % 32 == 0
    out = np.zeros((n // 32, m, bits), dtype=np.uint64)
    for c in range(n // 32):
        for j in range(32):
            pos = j * bits
            wi, sh = pos // 32, pos % 32
            v = codes[:, c * 32 + j].astype(np.uint64) << np.uint64(sh)
            out[c, :, wi] |= v & np.uint64(0xFFFFFFFF)
            if sh + bits > 32:
                out[c, :, wi + 1] |= v >> np.uint64(32)
    return out.astype(np.uint32)


def unpack_codes(packed: np.ndarray, bits: int, n: int) -> np.ndarray:
    chunks, m, _ = packed.shape
    assert chunks * 32 == n
    out = np.zeros((m, n), dtype=np.uint8)
    p64 = packed.astype(np.uint64)
    mask = np.uint64((1 << bits) - 1)
    for c in range(chunks):
        for j in range(32):
            pos = j * bits
            wi, sh = pos // 32, pos % 32
            v = p64[c, :, wi] >> np.uint64(sh)
            if sh + bits > 32:
                v |= p64[c, :, wi + 1] << np.uint64(32 - sh)
            out[:, c * 32 + j] = (v & mask).astype(np.uint8)
    return out


def dequantize(codes, scales, zeros, group: int) -> np.ndarray:
    """scale (code - zero), one scale and zero-point per (row, group of columns)."""
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    z = np.repeat(zeros.astype(np.float64), group, axis=1)
    return s * (codes.astype(np.float64) - z)


def low_rank_apply(X: np.ndarray, U_code, V_code, sigma, s) -> np.ndarray:
    """X W_r^T as two thin products: ((X diag(s)^-1) V^T diag(sigma)) U      (Eq. 3, 4)"""
    U = ro.e4m3_decode(U_code)
    V = ro.e4m3_decode(V_code)
    Y = (X.astype(np.float64) / s.astype(np.float64)[None, :]) @ V.T
    return (Y * np.asarray(sigma, dtype=np.float64)[None, :]) @ U


def linear_forward(X, packed, bits, scales, zeros, group, perm, b_I, b_H, U_code, V_code, sigma, s):
    """O = X~ Dequant(W_q)^T + low-rank part, X~ = X P Q                          (Eq. 7)"""
    n = X.shape[1]
    Xt = lo.rotate_weight(X.astype(np.float64), perm, b_I, b_H)       # rows of X times P Q
    Wq = dequantize(unpack_codes(packed, bits, n), scales, zeros, group)
    return Xt @ Wq.T + low_rank_apply(X, U_code, V_code, sigma, s)
