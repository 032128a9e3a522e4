"""CPU oracle for the layer-wise post-training quantization solve.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, double-precision numpy
implementation of the per-layer solve of  min || W X - Q(W) X ||_F  that the
GPU library is checked against.  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import it; the product path never does, and
it shares no code with the HIP kernels.

What the paper fixes (LoPRo, arXiv 2601.19675):
  * the objective and the proxy Hessian H = E[X X^T]       (Sec. 2, Eq. 1;
    restated for the rotated residual in Sec. 3.2, Eq. 8, and Algorithm 1);
  * that the quantizer walks over weight columns one after another and pushes
    each column's error onto the columns that follow      (Sec. 2, "Solution
    to O1", item (a));
  * group-wise scalar grids with one scale per group of 128 (Sec. 3.4, Eq. 12
    and the average-bit appendix).
Everything the paper leaves open is a stated reading (function docstrings):
raw-sum Hessian, relative damping, the Cholesky factor of the damped inverse
as compensation coefficients, min/max asymmetric grids that contain zero and
are taken from the row's current (already compensated) values when the column
loop enters the group, float32 scales, round-half-to-even.

The algorithm is a greedy heuristic, so the oracle is the recurrence itself,
column by column, with no blocking: block size and lazy batching of updates
are re-associations that change nothing in exact arithmetic.

Parity status of each function (what pins it, see tests/test_oracle_pins.py):
  hessian                 brute-force loops, closed forms
  damp                    closed form
  inverse_cholesky_upper  hand-computed 2x2 / 3x3 factors, U^T U H_d = I,
                          the reversed-Cholesky route (factor uniqueness)
  quantize_layer          on-grid recovery, diagonal-H = round-to-nearest,
                          conditional optimality against a least-squares
                          Schur complement, brute force on 1-4 columns,
                          (W - Wq) = E U  and  sum e^2 = tr(D H_d D^T)
  layer_error             trace identity against the X-side definition
"""
from __future__ import annotations

import numpy as np
import scipy.linalg


# ----------------------------------------------------------------------------
# step 1: proxy Hessian                                    (Sec. 2, Eq. 1)
# ----------------------------------------------------------------------------
def hessian(X: np.ndarray, H: np.ndarray | None = None, chunk: int = 16384) -> np.ndarray:
    """H (+)= X^T X for X given as tokens x channels in float64.

    Reading: the expectation in Eq. 1 is taken as the raw sum over calibration
    tokens (no 1/t, no factor 2); the solve is invariant to a positive rescale
    of H because the damping below is relative.  Tokens are consumed in slabs
    only to bound memory; the slabs are simply added.
    """
    t, n = X.shape
    if H is None:
        H = np.zeros((n, n), dtype=np.float64)
    for lo in range(0, t, chunk):
        xc = np.asarray(X[lo:lo + chunk], dtype=np.float64)
        H += xc.T @ xc
    return H


# ----------------------------------------------------------------------------
# step 2: dead channels, damping, factor of the inverse
# ----------------------------------------------------------------------------
def damp(H: np.ndarray, lam: float):
    """Returns (H_d, dead): H_d = H' + lam * mean(diag H') * I.

    Reading (paper silent): a channel that never fires (H_jj == 0) gets
    H'_jj = 1 and is reported in `dead` so that its weight column is zeroed
    before the solve; the mean of the diagonal is taken after that fix.
    """
    Hd = np.array(H, dtype=np.float64, copy=True)
    d = np.diag(Hd).copy()
    dead = d == 0.0
    d[dead] = 1.0
    np.fill_diagonal(Hd, d)
    Hd[np.diag_indices_from(Hd)] += lam * d.mean()
    return Hd, dead


def inverse_cholesky_upper(Hd: np.ndarray) -> np.ndarray:
    """The upper-triangular U with positive diagonal and U^T U = H_d^{-1}.

    Textbook route: Cholesky of H_d, explicit inverse, Cholesky of the inverse.
    Row j of U holds the coefficients with which the error of column j is
    pushed onto columns k > j.
    """
    Hd = np.asarray(Hd, dtype=np.float64)
    n = Hd.shape[0]
    L = np.linalg.cholesky(Hd)
    Linv = scipy.linalg.solve_triangular(L, np.eye(n), lower=True)
    Hinv = Linv.T @ Linv
    return np.linalg.cholesky(Hinv).T.copy()


# ----------------------------------------------------------------------------
# step 3: column-by-column quantize + compensate
# ----------------------------------------------------------------------------
def group_grid(wg: np.ndarray, maxq: int):
    """Asymmetric min/max grid of one group for every row of `wg` (rows x g).

    Reading: range forced to contain 0; degenerate range -> [-1, 1];
    scale = float32((max - min) / maxq) and that rounded value is the one used
    afterwards; zero = round_half_even(-min / scale), an integer in [0, maxq].
    Returns scale (float64 holding float32 values), zero (float64 integers),
    and the two pre-rounding values (range/maxq and -min/scale) for tie reports.
    """
    xmin = np.minimum(wg.min(axis=1), 0.0)
    xmax = np.maximum(wg.max(axis=1), 0.0)
    flat = xmin == xmax
    xmin = np.where(flat, -1.0, xmin)
    xmax = np.where(flat, 1.0, xmax)
    pre_scale = (xmax - xmin) / maxq
    scale = pre_scale.astype(np.float32).astype(np.float64)
    pre_zero = -xmin / scale
    zero = np.rint(pre_zero)
    return scale, zero, pre_scale, pre_zero, xmin


def quantize_layer(W: np.ndarray, U: np.ndarray, bits: int, group: int,
                   dead: np.ndarray | None = None, forced: dict | None = None,
                   want_pre: bool = False, static_groups: bool = False):
    """Greedy column-sequential quantization of the rows of W (m x n).

    For column j (Sec. 2, item (a): quantize a column, compensate the later
    ones):    code = clip(rne(w_j / scale) + zero, 0, maxq)
              q    = scale * (code - zero)
              e    = (w_j - q) / U_jj
              w_k -= e * U_jk      for every k > j.
    The grid of a group is taken from the row's current values when j reaches
    the first column of that group, or -- `static_groups`, an option of the
    quantizer the paper names in that item -- from the row's values as they
    were handed over, before any compensation.

    `forced` (used by the parity protocol for near-ties) maps
    ("code", r, j) / ("zero", r, k) / ("scale", r, k) to the value to take
    instead of the computed one.

    Returns a dict: codes (uint8 m x n), scales (float32 m x n/g), zeros
    (uint8 m x n/g), Wq (float64), E (float64, the e's), row_err2 (sum_j e^2),
    and, when want_pre, the pre-rounding values x = w_j/scale (m x n),
    pre_zero and pre_scale (m x n/g) used to recognise near-ties.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    m, n = W.shape
    assert n % group == 0 and 2 <= bits <= 8
    maxq = float(2 ** bits - 1)
    ng = n // group
    if dead is not None:
        W[:, np.asarray(dead, dtype=bool)] = 0.0
    W_given = W.copy()
    forced = forced or {}
    f_code, f_zero, f_scale = {}, {}, {}
    for (kind, r, idx), v in forced.items():
        {"code": f_code, "zero": f_zero, "scale": f_scale}[kind].setdefault(idx, []).append((r, v))

    codes = np.zeros((m, n), dtype=np.uint8)
    scales = np.zeros((m, ng), dtype=np.float32)
    zeros = np.zeros((m, ng), dtype=np.uint8)
    Wq = np.zeros((m, n))
    E = np.zeros((m, n))
    pre_x = np.zeros((m, n)) if want_pre else None
    pre_z = np.zeros((m, ng)) if want_pre else None
    pre_s = np.zeros((m, ng)) if want_pre else None
    scale = zero = None
    for j in range(n):
        if j % group == 0:
            k = j // group
            scale, zero, ps, pz, xmin = group_grid((W_given if static_groups else W)[:, j:j + group], int(maxq))
            if k in f_scale:
                for r, v in f_scale[k]:
                    scale[r] = float(np.float32(v))
                    pz[r] = -xmin[r] / scale[r]
                    zero[r] = np.rint(pz[r])
            if k in f_zero:
                for r, v in f_zero[k]:
                    zero[r] = float(v)
            scales[:, k] = scale.astype(np.float32)
            zeros[:, k] = zero.astype(np.uint8)
            if want_pre:
                pre_s[:, k] = ps
                pre_z[:, k] = pz
        w = W[:, j]
        x = w / scale
        c = np.clip(np.rint(x) + zero, 0.0, maxq)
        if j in f_code:
            for r, v in f_code[j]:
                c[r] = float(v)
        q = scale * (c - zero)
        e = (w - q) / U[j, j]
        if j + 1 < n:
            W[:, j + 1:] -= np.outer(e, U[j, j + 1:])
        codes[:, j] = c.astype(np.uint8)
        Wq[:, j] = q
        E[:, j] = e
        if want_pre:
            pre_x[:, j] = x
    out = dict(codes=codes, scales=scales, zeros=zeros, Wq=Wq, E=E,
               row_err2=(E * E).sum(axis=1))
    if want_pre:
        out.update(pre_x=pre_x, pre_zero=pre_z, pre_scale=pre_s)
    return out


def round_to_nearest(W: np.ndarray, bits: int, group: int):
    """Per-group min/max rounding with no compensation (the RTN baseline of the
    paper's ablation, Sec. 4.4, Tab. 5): the same grids taken from W itself."""
    W = np.asarray(W, dtype=np.float64)
    m, n = W.shape
    maxq = 2 ** bits - 1
    codes = np.zeros((m, n), dtype=np.uint8)
    Wq = np.zeros((m, n))
    scales = np.zeros((m, n // group), dtype=np.float32)
    zeros = np.zeros((m, n // group), dtype=np.uint8)
    for k in range(n // group):
        sl = slice(k * group, (k + 1) * group)
        scale, zero, _, _, _ = group_grid(W[:, sl], maxq)
        c = np.clip(np.rint(W[:, sl] / scale[:, None]) + zero[:, None], 0, maxq)
        codes[:, sl] = c.astype(np.uint8)
        Wq[:, sl] = scale[:, None] * (c - zero[:, None])
        scales[:, k] = scale.astype(np.float32)
        zeros[:, k] = zero.astype(np.uint8)
    return dict(codes=codes, scales=scales, zeros=zeros, Wq=Wq)


def dequantize(codes, scales, zeros, group: int) -> np.ndarray:
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    z = np.repeat(zeros.astype(np.float64), group, axis=1)
    return s * (codes.astype(np.float64) - z)


# ----------------------------------------------------------------------------
# step 4: layer error                                       (Sec. 2, Eq. 1)
# ----------------------------------------------------------------------------
def layer_error(W: np.ndarray, Wq: np.ndarray, H: np.ndarray):
    """(rel, num, den): rel = sqrt(tr(D H D^T) / tr(W H W^T)), D = W - Wq,
    with the undamped H and the original W; equals ||WX - QX||_F / ||WX||_F."""
    W = np.asarray(W, dtype=np.float64)
    D = W - np.asarray(Wq, dtype=np.float64)
    num = float(np.einsum("ij,ij->", D @ H, D))
    den = float(np.einsum("ij,ij->", W @ H, W))
    return float(np.sqrt(num / den)), num, den


def layer_error_from_activations(W: np.ndarray, Wq: np.ndarray, X: np.ndarray):
    """The same ratio straight from its definition, X given tokens x channels."""
    W = np.asarray(W, dtype=np.float64)
    Y = X @ W.T
    Yq = X @ np.asarray(Wq, dtype=np.float64).T
    return float(np.linalg.norm(Y - Yq) / np.linalg.norm(Y))


def symmetrize_from_upper(Hu: np.ndarray) -> np.ndarray:
    """Full symmetric matrix from one whose upper triangle is defined."""
    T = np.triu(Hu)
    return T + np.triu(Hu, 1).T
