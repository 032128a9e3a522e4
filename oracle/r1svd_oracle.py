"""CPU oracle for LoPRo's scaled rank-one randomized low-rank step (R1SVD).

TEST INFRASTRUCTURE ONLY (see ptq_oracle.py): plain float64 numpy, one matrix-vector
product per line, the matrix deflated in place exactly as the algorithm box states.
Nothing here is imported by the product path and no code is shared with the HIP kernels.

What the paper fixes (LoPRo, arXiv 2601.19675):
  * the activation scale (Algorithm 1):  Xbar = mean(|X|, axis=0),
        s = Xbar^2.5 / sqrt(max(Xbar) * min(Xbar)),      W_s = W diag(s);
  * one rank-one step on the current matrix A (Sec. 3.3, Eq. 9-11; Algorithm 1):
        y = (A A^T)^it A v,   p = A^T y,
        U_1 = y / ||y||,  V_1 = p / ||p||,  sigma = ||p|| / ||y||,
    followed by the deflation A <- A - sigma U_1 V_1^T and the next rank;
  * U and V are kept in 8-bit floating point, e4m3, Sigma in fp16 (Sec. 3.3 and the
    implementation details appendix), and the rounding error of one rank is left in the
    deflated matrix for the later ranks to pick up;
  * r = 16 and it = 8 in the paper's runs;
  * the residual handed to the quantizer:  R = A_final diag(s)^-1   (Algorithm 1).

Readings (the text leaves these open):
  * e4m3 is the OCP 8-bit format (4 exponent bits with bias 7, 3 mantissa bits, subnormals
    with quantum 2^-9, largest finite value 448, no infinities); conversion rounds to nearest,
    ties to even, and saturates.  The paper names the format but no rounding mode.
  * The deflation uses the STORED values (U_1 and V_1 after rounding to e4m3, sigma after
    rounding to fp16): that is what makes later ranks compensate the rounding, and it makes
    W_s = A_final + sum_k sigma_k U_k V_k^T hold exactly for what is stored.
  * The random vector v is an input (standard normal draws in the tests), one per rank.
  * The algorithm box counts "2 + iter" matrix-vector products; the formula it prints needs
    2 + 2 iter.  The formula is followed.
  * Scaling y between the products would change nothing (U_1, V_1 and sigma are ratios);
    the oracle applies the printed formula as it stands.
  * If y or p is the zero vector the step stores U_1 = V_1 = 0 and sigma = 0.
  * sigma can exceed the fp16 range (65504) when the activation scale is large; an IEEE
    conversion would store infinity and destroy the matrix at the deflation.  The conversion
    saturates at 65504: the deflation then removes only part of that direction and the next
    ranks find the rest, which is the compensation mechanism the paper relies on anyway.
  * A channel that is never active (Xbar_j = 0) would make the printed scale 0/0 or
    divide by zero for every channel: max and min run over the positive entries and such
    a channel gets s_j = 1.

Parity status (tests/test_r1svd_oracle_pins.py): the e4m3 rounding and its 256 code
values against torch's float8_e4m3fn conversion; the scale against a hand-worked example,
its closed form for constant Xbar and its degree of homogeneity; one rank-one step against
the closed form for an exactly rank-one matrix, against numpy's SVD (leading triplet of a
matrix with a spectral gap), and against the definition with an explicit matrix power; the
whole loop against the Eckart-Young bound, the reconstruction identity, and the residual's
orthogonality to the stored factors in the unrounded mode.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0
_E4M3_MIN_EXP = -6          # exponent of the smallest normal number
_E4M3_MANT_BITS = 3


def mean_abs_activation(X: np.ndarray) -> np.ndarray:
    """Xbar = mean(|X|, axis=0)                                       (Algorithm 1)"""
    return np.mean(np.abs(X.astype(np.float64)), axis=0)


def activation_scale(xbar: np.ndarray) -> np.ndarray:
    """s = Xbar^2.5 / sqrt(max(Xbar) min(Xbar))                       (Algorithm 1)"""
    xbar = xbar.astype(np.float64)
    live = xbar > 0.0
    s = np.ones_like(xbar)
    if np.any(live):
        hi = np.max(xbar[live])
        lo = np.min(xbar[live])
        s[live] = xbar[live] ** 2.5 / np.sqrt(hi * lo)
    return s


def e4m3_round(x: np.ndarray):
    """Nearest e4m3 value (ties to even, saturating) and the distance to the rounding tie.

    Returns (value, margin): margin is |frac - 0.5| of x in units of the local quantum, i.e.
    0 means x sits exactly between two representable values.
    """
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    _, ex = np.frexp(a)                       # a = f * 2^ex, f in [0.5, 1)
    e = np.maximum(ex - 1, _E4M3_MIN_EXP)     # binade of a, clamped into the subnormal range
    quantum = np.ldexp(1.0, e - _E4M3_MANT_BITS)
    t = a / quantum
    r = np.rint(t)                            # numpy rounds halves to even
    margin = np.abs(np.abs(t - np.floor(t)) - 0.5)
    val = np.minimum(r * quantum, E4M3_MAX)
    margin = np.where(a >= E4M3_MAX, 0.5, margin)
    return np.copysign(val, x), margin


def e4m3_encode(val: np.ndarray) -> np.ndarray:
    """Byte codes (sign, 4 exponent bits, 3 mantissa bits) of values e4m3_round returned."""
    val = np.asarray(val, dtype=np.float64)
    a = np.abs(val)
    _, ex = np.frexp(a)
    e = ex - 1
    normal = a >= np.ldexp(1.0, _E4M3_MIN_EXP)
    sub_code = np.rint(a / np.ldexp(1.0, _E4M3_MIN_EXP - _E4M3_MANT_BITS)).astype(np.int64)
    mant = np.rint((a / np.ldexp(1.0, e) - 1.0) * 8.0).astype(np.int64)
    norm_code = ((e + 7) << 3) | mant
    code = np.where(normal, norm_code, sub_code)
    code = code | (np.signbit(val).astype(np.int64) << 7)
    return code.astype(np.uint8)


def e4m3_decode(code: np.ndarray) -> np.ndarray:
    """Value of each byte code (0x7f / 0xff, the NaN codes, never occur here)."""
    c = np.asarray(code).astype(np.int64)
    ef = (c >> 3) & 0xF
    m = c & 0x7
    mag = np.where(ef == 0, m * np.ldexp(1.0, -9), (1.0 + m / 8.0) * np.ldexp(1.0, ef - 7))
    return np.where(c & 0x80, -mag, mag)


FP16_MAX = 65504.0


def fp16_round(x: float) -> float:
    """Nearest fp16 value, ties to even; beyond the format's range the largest finite value."""
    return float(np.float16(min(x, FP16_MAX)))


def _quantum(x: np.ndarray, min_exp: int, mant_bits: int) -> np.ndarray:
    """Spacing of the format's values in the binade of |x|."""
    _, ex = np.frexp(np.abs(np.asarray(x, dtype=np.float64)))
    return np.ldexp(1.0, np.maximum(ex - 1, min_exp) - mant_bits)


def rank_one_step(A: np.ndarray, v: np.ndarray, it: int):
    """y, p of Algorithm 1 and the unrounded triplet (U_1, sigma, V_1)      (Eq. 11)"""
    y = A @ v
    for _ in range(it):
        y = A @ (A.T @ y)
    p = A.T @ y
    ny = float(np.sqrt(np.sum(y * y)))
    nump = float(np.sqrt(np.sum(p * p)))
    if ny == 0.0 or nump == 0.0:
        return np.zeros_like(y), 0.0, np.zeros_like(p)
    return y / ny, nump / ny, p / nump


def r1svd(A: np.ndarray, S: np.ndarray, it: int, rounded: bool = True,
          U_force: np.ndarray | None = None, V_force: np.ndarray | None = None,
          sigma_force: np.ndarray | None = None):
    """Rank-by-rank sketch of A with deflation (Sec. 3.3; Algorithm 1, inner loop).

    S is r x n, one sketch vector per rank.  With `rounded` the factors are stored in
    e4m3 / fp16 and the stored values are what is deflated.  U_force / V_force (r x m,
    r x n, int16, -1 = no override) replace single codes and sigma_force (r, NaN = no
    override) a stored sigma: a parity protocol uses them where a value sits on a rounding
    tie, so that one flipped code does not hide everything after it.

    Returns dict: U (r x m), V (r x n), sigma (r) as stored values (float64), U_code,
    V_code (uint8, only with `rounded`), U_margin, V_margin, the unrounded U_exact, V_exact,
    sigma_exact of every rank (given the earlier ranks as stored), and A (the deflated matrix).
    """
    A = np.array(A, dtype=np.float64, copy=True)
    m, n = A.shape
    r = S.shape[0]
    U = np.zeros((r, m)); V = np.zeros((r, n)); sig = np.zeros(r)
    Ue = np.zeros((r, m)); Ve = np.zeros((r, n)); sige = np.zeros(r)
    Uc = np.zeros((r, m), dtype=np.uint8); Vc = np.zeros((r, n), dtype=np.uint8)
    Um = np.full((r, m), 0.5); Vm = np.full((r, n), 0.5)
    for k in range(r):
        u, sg, vv = rank_one_step(A, S[k].astype(np.float64), it)
        Ue[k], Ve[k], sige[k] = u, vv, sg
        if rounded:
            u, Um[k] = e4m3_round(u)
            vv, Vm[k] = e4m3_round(vv)
            Uc[k] = e4m3_encode(u)
            Vc[k] = e4m3_encode(vv)
            if U_force is not None:
                f = U_force[k] >= 0
                Uc[k][f] = U_force[k][f].astype(np.uint8)
                u = e4m3_decode(Uc[k])
            if V_force is not None:
                f = V_force[k] >= 0
                Vc[k][f] = V_force[k][f].astype(np.uint8)
                vv = e4m3_decode(Vc[k])
            sg = fp16_round(sg)
            if sigma_force is not None and not np.isnan(sigma_force[k]):
                sg = float(sigma_force[k])
        U[k], V[k], sig[k] = u, vv, sg
        A -= sg * np.outer(u, vv)
    return {"U": U, "V": V, "sigma": sig, "U_code": Uc, "V_code": Vc, "U_margin": Um, "V_margin": Vm,
            "U_exact": Ue, "V_exact": Ve, "sigma_exact": sige, "A": A}


def quantum(x: np.ndarray, fmt: str) -> np.ndarray:
    """Spacing of the stored format's values ("e4m3" or "fp16") in the binade of |x|."""
    if fmt == "e4m3":
        return _quantum(x, _E4M3_MIN_EXP, _E4M3_MANT_BITS)
    if fmt == "fp16":
        return _quantum(x, -14, 10)
    raise ValueError(fmt)


def scaled_r1svd(W: np.ndarray, s: np.ndarray, S: np.ndarray, it: int, rounded: bool = True,
                 U_force: np.ndarray | None = None, V_force: np.ndarray | None = None,
                 sigma_force: np.ndarray | None = None):
    """W_s = W diag(s), its sketch, and the residual R = A diag(s)^-1       (Algorithm 1)"""
    s = s.astype(np.float64)
    out = r1svd(W.astype(np.float64) * s[None, :], S, it, rounded, U_force, V_force, sigma_force)
    out["R"] = out["A"] / s[None, :]
    return out


def low_rank_weight(out: dict, s: np.ndarray) -> np.ndarray:
    """W_r = (U Sigma)(V diag(s)^-1), the part kept in high precision       (Eq. 4)"""
    return (out["U"].T * out["sigma"][None, :]) @ (out["V"] / s.astype(np.float64)[None, :])
