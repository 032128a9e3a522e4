"""CPU oracle for LoPRo's pre-conditioning of the layer solve: column permutation and
partial block Walsh-Hadamard rotation of the residual and of the proxy Hessian.

TEST INFRASTRUCTURE ONLY (see ptq_oracle.py): plain float64 numpy, dense matrices, no
fast transform -- Q and P are built explicitly and multiplied out, so that every line can
be held against the paper's formulas.  Nothing here is imported by the product path and
no code is shared with the HIP kernels.

What the paper fixes (LoPRo, arXiv 2601.19675, Sec. 3.2 and Algorithm 1):
  * the ranking key  diag(H) / amean(R, axis=0)  of a column (Eq. 5), amean = mean of the
    absolute values down a column;
  * the partial rotation  Q = blockdiag(I_{b_I}, H_wal, .., H_wal)  with H_wal a
    b_H x b_H Walsh-Hadamard matrix, b_H a power of two, and  R' = R P Q  (Eq. 6);
  * the Hessian that goes with the rotated residual,  H' = Q^T P^T H P Q  (Eq. 8), and
    the way back,  W = W_r + Q(R') Q^T P^T  (Eq. 7);
  * b_I = b_H = 256 in all experiments (implementation details appendix).

Readings (the text leaves these open or is at odds with itself):
  * H_wal is the Sylvester (natural-order) Hadamard matrix scaled by 1/sqrt(b_H), so that
    Q^T Q = I as the proofs assume; for b_H = 256 the scale 1/16 is exact.
  * P applies `perm` as a gather: column c of R P is column perm[c] of R, i.e.
    P[perm[c], c] = 1.  (Read literally, "P_{i,perm[i]} = 1" with perm an argsort would
    scatter, which orders nothing.)
  * Direction: Eq. 5 says ascending sort, the prose says that important columns (small
    |R|, hence LARGE key) and columns with large diag(H) come first.  The prose is what
    the identity block is for, so the default is descending keys; `descending=False`
    gives the literal ascending order.  Ties keep the lower index first.  A column whose
    amean is zero gets key +inf if diag(H) > 0 and 0 otherwise (0/0).
  * (n - b_I) must be a multiple of b_H.

Parity status (tests/test_lopro_oracle_pins.py): column_keys against a hand-worked
example; permutation against a hand-worked example and sortedness; hadamard against
scipy.linalg.hadamard and orthogonality; rotation against the loss invariance of Eq. 8 /
Theorem 2, the identity of Eq. 7, orthogonality (exact round trip on dyadic inputs),
spectrum and trace of H', and the untouched identity block.
"""
from __future__ import annotations

import numpy as np


def column_keys(H: np.ndarray, R: np.ndarray) -> np.ndarray:
    """diag(H) / amean(R, axis=0)                                     (Sec. 3.2, Eq. 5)"""
    d = np.diag(H).astype(np.float64)
    a = np.mean(np.abs(R.astype(np.float64)), axis=0)
    keys = np.empty_like(d)
    nz = a != 0.0
    keys[nz] = d[nz] / a[nz]
    keys[~nz] = np.where(d[~nz] > 0.0, np.inf, 0.0)
    return keys


def permutation(keys: np.ndarray, descending: bool = True) -> np.ndarray:
    """perm = sort(keys).idx (Eq. 5); ties keep the lower column index first."""
    n = keys.shape[0]
    order = sorted(range(n), key=(lambda j: (-keys[j], j)) if descending else (lambda j: (keys[j], j)))
    return np.asarray(order, dtype=np.int64)


def permutation_matrix(perm: np.ndarray) -> np.ndarray:
    """P with (R P)[:, c] = R[:, perm[c]]."""
    n = perm.shape[0]
    P = np.zeros((n, n), dtype=np.float64)
    P[perm, np.arange(n)] = 1.0
    return P


def hadamard(b: int) -> np.ndarray:
    """Sylvester Hadamard matrix of order b (a power of two), scaled to be orthogonal."""
    assert b >= 1 and (b & (b - 1)) == 0
    Hm = np.ones((1, 1), dtype=np.float64)
    while Hm.shape[0] < b:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    return Hm / np.sqrt(float(b))


def rotation_matrix(n: int, b_I: int, b_H: int) -> np.ndarray:
    """Q = blockdiag(I_{b_I}, H_wal, .., H_wal)                        (Sec. 3.2, Eq. 6)"""
    assert 0 <= b_I <= n and (n - b_I) % b_H == 0
    Q = np.zeros((n, n), dtype=np.float64)
    Q[:b_I, :b_I] = np.eye(b_I)
    Hw = hadamard(b_H)
    for s in range(b_I, n, b_H):
        Q[s:s + b_H, s:s + b_H] = Hw
    return Q


def rotate_weight(R: np.ndarray, perm: np.ndarray, b_I: int, b_H: int) -> np.ndarray:
    """R' = R P Q                                                      (Eq. 6)"""
    n = R.shape[1]
    return R.astype(np.float64) @ permutation_matrix(perm) @ rotation_matrix(n, b_I, b_H)


def unrotate_weight(Rq: np.ndarray, perm: np.ndarray, b_I: int, b_H: int) -> np.ndarray:
    """Q(R') Q^T P^T: the quantized residual back in the layer's own basis   (Eq. 7)"""
    n = Rq.shape[1]
    return Rq.astype(np.float64) @ rotation_matrix(n, b_I, b_H).T @ permutation_matrix(perm).T


def rotate_hessian(H: np.ndarray, perm: np.ndarray, b_I: int, b_H: int) -> np.ndarray:
    """H' = Q^T P^T H P Q                                              (Eq. 8)"""
    n = H.shape[0]
    P = permutation_matrix(perm)
    Q = rotation_matrix(n, b_I, b_H)
    return Q.T @ (P.T @ H.astype(np.float64) @ P) @ Q
