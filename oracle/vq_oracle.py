"""CPU oracle for the vector-quantized variant of the column solve (LoPRo_v).

TEST INFRASTRUCTURE ONLY (see ptq_oracle.py): plain float64 numpy, one group of columns at
a time, no blocking.  Nothing here is imported by the product path and no code is shared
with the HIP kernels.

What the paper fixes (LoPRo, arXiv 2601.19675; implementation-details appendix; Sec. 3.2,
Eq. 8; Algorithm 1, the quantization step, which may be a scalar or a vector quantizer):
  * the vector variant uses the simplest form of vector quantization: a codebook that is
    drawn at random and never trained, no block-wise scaling of the weights;
  * vectors of 4 consecutive weights at 2 bits per weight (an 8-bit index, 256 entries) and
    of 2 consecutive weights at 3 bits per weight (a 6-bit index, 64 entries);
  * the assignment minimises the same proxy-Hessian loss as the scalar solve (Eq. 8), and
    the error of what has been assigned is compensated in the columns that follow (Sec. 2,
    item (a), carried over from the scalar quantizer).

Readings (the text leaves these open):
  * The codebook is an INPUT: K x d values in the weights' own units, one codebook for the
    whole layer.  How it is drawn is the caller's business (the tests draw entries from the
    layer's own d-column pieces); granularity finer than a layer is not covered.
  * A vector is d consecutive columns of one row, starting at a multiple of d.
  * With U the upper factor of the damped inverse Hessian (as in the scalar solve) and
    T = U[j:j+d, j:j+d], the errors of the d columns of a group, taken one after the other as
    the scalar solve would, are  e = (w - c) T^-1  (forward substitution), and the loss the
    group adds -- with the earlier columns fixed and the later ones left continuous -- is
    sum_i e_i^2.  The entry with the smallest such sum is assigned; among entries with exactly
    equal sums the lowest index wins.
  * Then  w_k -= sum_i e_i U[j+i, k]  for every later column k, as in the scalar solve.
  * A dead channel's weight column counts as zero.

Parity status (tests/test_vq_oracle_pins.py): d = 1 against a scalar nearest-entry walk
written with Python scalars; a diagonal Hessian against the plain weighted nearest-neighbour
search on the weights as given; conditional optimality of every group against a Schur
complement of H_d that never touches U; brute force over all K^(n/d) assignments of tiny
layers; exact recovery of weights made of codebook entries; the error identities
(W - Wq) = E U and sum e^2 = tr(D H_d D^T); invariance under a permutation of the codebook.
"""
from __future__ import annotations

import numpy as np


def group_errors(w: np.ndarray, c: np.ndarray, T: np.ndarray) -> np.ndarray:
    """e = (w - c) T^-1 by forward substitution, for rows w (r x d) against one entry c (d):
    the errors of the group's columns taken one after the other."""
    d = T.shape[0]
    rem = w - c[None, :]
    e = np.zeros_like(rem)
    for i in range(d):
        e[:, i] = rem[:, i] / T[i, i]
        for k in range(i + 1, d):
            rem[:, k] -= e[:, i] * T[i, k]
    return e


def quantize_layer_vq(W: np.ndarray, U: np.ndarray, codebook: np.ndarray, dead: np.ndarray | None = None,
                      forced: dict | None = None, want_margins: bool = False):
    """Greedy group-sequential vector quantization of the rows of W (m x n) with compensation.

    codebook: K x d.  `forced` maps (row, group) -> index to take instead of the computed one (the
    parity protocol uses it at near-ties).  Returns a dict: indices (m x n/d, int32), Wq, E
    (the e's, m x n), row_err2, and with want_margins the loss of the assigned entry (best), the
    second-smallest loss (second) of every (row, group) and pre_w (m x n), the compensated values
    each group had when it was assigned; group_losses() below recomputes all K losses of one
    group from them for a caller that needs more than the two smallest.
    """
    W = np.array(W, dtype=np.float64, copy=True)
    C = np.asarray(codebook, dtype=np.float64)
    K, d = C.shape
    m, n = W.shape
    assert n % d == 0
    if dead is not None:
        W[:, np.asarray(dead, dtype=bool)] = 0.0
    forced = forced or {}
    ng = n // d
    idx = np.zeros((m, ng), dtype=np.int32)
    Wq = np.zeros((m, n))
    E = np.zeros((m, n))
    best = np.zeros((m, ng)) if want_margins else None
    second = np.zeros((m, ng)) if want_margins else None
    pre_w = np.zeros((m, n)) if want_margins else None
    for g in range(ng):
        j = g * d
        T = U[j:j + d, j:j + d]
        w = W[:, j:j + d]
        loss = np.empty((m, K))
        for k in range(K):
            e = group_errors(w, C[k], T)
            loss[:, k] = np.sum(e * e, axis=1)
        choice = np.argmin(loss, axis=1)            # the lowest index among equal losses
        for (r, gg), v in forced.items():
            if gg == g:
                choice[r] = int(v)
        if want_margins:
            srt = np.sort(loss, axis=1)
            best[:, g] = loss[np.arange(m), choice]
            second[:, g] = srt[:, 1] if K > 1 else np.inf
            pre_w[:, j:j + d] = w
        q = C[choice]
        e = np.zeros((m, d))
        rem = w - q
        for i in range(d):
            e[:, i] = rem[:, i] / T[i, i]
            for k in range(i + 1, d):
                rem[:, k] -= e[:, i] * T[i, k]
        if j + d < n:
            W[:, j + d:] -= e @ U[j:j + d, j + d:]
        idx[:, g] = choice
        Wq[:, j:j + d] = q
        E[:, j:j + d] = e
    out = dict(indices=idx, Wq=Wq, E=E, row_err2=(E * E).sum(axis=1))
    if want_margins:
        out.update(best=best, second=second, pre_w=pre_w)
    return out


def group_losses(w: np.ndarray, codebook: np.ndarray, T: np.ndarray) -> np.ndarray:
    """All K losses of one row's group values w (d) -- what the assignment compares."""
    C = np.asarray(codebook, dtype=np.float64)
    return np.array([float(np.sum(group_errors(w[None, :], C[k], T) ** 2)) for k in range(C.shape[0])])


def nearest_entries(W: np.ndarray, codebook: np.ndarray) -> np.ndarray:
    """Plain vector quantization with no Hessian and no compensation: every d-column piece of W
    goes to its Euclidean-nearest entry (the vector analogue of round-to-nearest)."""
    W = np.asarray(W, dtype=np.float64)
    C = np.asarray(codebook, dtype=np.float64)
    K, d = C.shape
    m, n = W.shape
    P = W.reshape(m, n // d, d)
    dist = ((P[:, :, None, :] - C[None, None, :, :]) ** 2).sum(axis=3)
    return np.argmin(dist, axis=2).astype(np.int32)
