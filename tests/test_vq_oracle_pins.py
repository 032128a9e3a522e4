"""Pins of the vector-quantized solve's oracle (oracle/vq_oracle.py): special cases that reduce
to a plain nearest-neighbour search, optimality statements that never touch the factor U, brute
force on tiny layers, and the error identities of the compensation (Sec. 3.2, Eq. 8; Sec. 2, item
(a); implementation-details appendix of the paper for the vector form)."""
import itertools

import numpy as np
import pytest

from oracle import ptq_oracle as orc
from oracle import vq_oracle as vq


def _spd(rng, n, t=None):
    t = t or 3 * n
    X = rng.standard_normal((t, n)) @ (np.eye(n) + 0.6 * rng.standard_normal((n, n)) / np.sqrt(n))
    X *= np.exp(rng.normal(0, 0.7, n))[None, :]
    H = X.T @ X
    Hd, _ = orc.damp(H, 0.01)
    return H, Hd, orc.inverse_cholesky_upper(Hd)


def test_one_dimensional_vectors_are_the_scalar_nearest_entry_walk():
    # d = 1: a "vector" is one weight, the loss of an entry is ((w - c) / U_jj)^2, so the walk is: nearest
    # entry, e = (w - q) / U_jj, push -- written here with Python scalars on one row at a time
    rng = np.random.default_rng(1)
    n, m = 12, 5
    _, _, U = _spd(rng, n)
    W = rng.standard_normal((m, n))
    C = np.sort(rng.standard_normal(7))[:, None]
    out = vq.quantize_layer_vq(W, U, C)
    for r in range(m):
        w = [float(x) for x in W[r]]
        for j in range(n):
            k = min(range(7), key=lambda kk: (abs(w[j] - float(C[kk, 0])), kk))
            assert out["indices"][r, j] == k
            e = (w[j] - float(C[k, 0])) / float(U[j, j])
            assert out["E"][r, j] == pytest.approx(e, rel=1e-12, abs=1e-300)
            for c in range(j + 1, n):
                w[c] -= e * float(U[j, c])


@pytest.mark.parametrize("d,K", [(2, 16), (4, 32)])
def test_diagonal_hessian_is_the_weighted_nearest_neighbour_of_the_given_weights(d, K):
    # H diagonal => U diagonal => nothing is pushed and the loss of an entry is sum_i (w_i - c_i)^2 H_ii
    rng = np.random.default_rng(2 + d)
    n, m = 8 * d, 9
    h = np.exp(rng.normal(0, 1, n))
    U = np.diag(1.0 / np.sqrt(h))
    W = rng.standard_normal((m, n))
    C = rng.standard_normal((K, d))
    out = vq.quantize_layer_vq(W, U, C)
    P = W.reshape(m, n // d, d)
    Hg = h.reshape(n // d, d)
    dist = (((P[:, :, None, :] - C[None, None]) ** 2) * Hg[None, :, None, :]).sum(axis=3)
    assert np.array_equal(out["indices"], np.argmin(dist, axis=2))
    # and with H = I it is the plain Euclidean search
    out1 = vq.quantize_layer_vq(W, np.eye(n), C)
    assert np.array_equal(out1["indices"], vq.nearest_entries(W, C))
    assert np.array_equal(out1["Wq"], C[out1["indices"]].reshape(m, n))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_every_group_is_conditionally_optimal(seed):
    """Given the entries already assigned to earlier groups and the later columns left free, the loss
    tr(D H_d D^T) as a function of this group's deviation delta is delta S^-1 delta^T + const with
    S = (H_d^-1)[g, g] - ... computed here from H_d alone: minimising over the later columns leaves the
    Schur complement H_d[a:, a:] / H_d[b:, b:] on the group, and the earlier groups shift its centre."""
    rng = np.random.default_rng(10 + seed)
    d, K, n, m = 2, 6, 8, 4
    _, Hd, U = _spd(rng, n)
    W = rng.standard_normal((m, n))
    C = rng.standard_normal((K, d))
    out = vq.quantize_layer_vq(W, U, C)
    for r in range(m):
        for g in range(n // d):
            a, b = g * d, (g + 1) * d
            # deviation of the earlier columns is fixed; choose this group's entry, then let the later
            # columns take their optimal continuous values: minimise D H_d D^T over D[b:] for each candidate
            losses = []
            for k in range(K):
                D = np.zeros(n)
                D[:a] = W[r, :a] - out["Wq"][r, :a]
                D[a:b] = W[r, a:b] - C[k]
                if b < n:
                    D[b:] = -np.linalg.solve(Hd[b:, b:], Hd[b:, :b] @ D[:b])
                losses.append(float(D @ Hd @ D))
            assert int(np.argmin(losses)) == out["indices"][r, g]


def test_brute_force_over_all_assignments_of_tiny_layers():
    rng = np.random.default_rng(5)
    d, K, n = 2, 3, 6
    _, Hd, U = _spd(rng, n)
    C = rng.standard_normal((K, d))
    worse = 0
    for trial in range(6):
        w = rng.standard_normal(n)
        out = vq.quantize_layer_vq(w[None, :], U, C)
        greedy = float((w - out["Wq"][0]) @ Hd @ (w - out["Wq"][0]))
        best = min(float((w - C[list(a)].reshape(-1)) @ Hd @ (w - C[list(a)].reshape(-1)))
                   for a in itertools.product(range(K), repeat=n // d))
        assert greedy >= best * (1 - 1e-12)
        worse += greedy > best * (1 + 1e-9)
    # one group: the greedy choice IS the optimum
    w = rng.standard_normal(d)
    _, Hd2, U2 = _spd(rng, d)
    out = vq.quantize_layer_vq(w[None, :], U2, C)
    losses = [float((w - C[k]) @ Hd2 @ (w - C[k])) for k in range(K)]
    assert out["indices"][0, 0] == int(np.argmin(losses))


def test_weights_made_of_codebook_entries_are_recovered_exactly():
    rng = np.random.default_rng(6)
    d, K, n, m = 4, 20, 16, 7
    _, _, U = _spd(rng, n)
    C = rng.standard_normal((K, d))
    idx = rng.integers(0, K, size=(m, n // d))
    W = C[idx].reshape(m, n)
    out = vq.quantize_layer_vq(W, U, C)
    assert np.array_equal(out["indices"], idx) and np.array_equal(out["Wq"], W) and not out["E"].any()


def test_error_identities_and_codebook_permutation():
    rng = np.random.default_rng(7)
    d, K, n, m = 4, 16, 24, 6
    _, Hd, U = _spd(rng, n)
    W = rng.standard_normal((m, n))
    C = rng.standard_normal((K, d))
    out = vq.quantize_layer_vq(W, U, C, want_margins=True)
    D = W - out["Wq"]
    assert np.allclose(D, out["E"] @ U, rtol=0, atol=1e-12)
    assert np.allclose(np.einsum("ij,ij->i", D @ Hd, D), out["row_err2"], rtol=1e-10)
    assert np.all(out["best"] <= out["second"])
    # the group's recorded loss is the sum of its squared errors
    assert np.allclose(out["best"], (out["E"] ** 2).reshape(m, n // d, d).sum(axis=2), rtol=1e-12)
    perm = rng.permutation(K)
    out2 = vq.quantize_layer_vq(W, U, C[perm])
    assert np.array_equal(out2["Wq"], out["Wq"]) and np.array_equal(perm[out2["indices"]], out["indices"])
    # a dead column counts as zero; a forced index is taken and compensated
    dead = np.zeros(n, dtype=bool); dead[5] = True
    Wz = W.copy(); Wz[:, 5] = 0.0
    assert np.array_equal(vq.quantize_layer_vq(W, U, C, dead=dead)["indices"], vq.quantize_layer_vq(Wz, U, C)["indices"])
    other = (int(out["indices"][2, 1]) + 1) % K
    f = vq.quantize_layer_vq(W, U, C, forced={(2, 1): other})
    assert f["indices"][2, 1] == other and np.array_equal(f["indices"][[0, 1, 3, 4, 5]], out["indices"][[0, 1, 3, 4, 5]])
    assert np.allclose(W[2] - f["Wq"][2], f["E"][2] @ U, atol=1e-12)


def test_exact_ties_take_the_lowest_index():
    C = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 0.0]])     # entries 0 and 2 are the same vector
    out = vq.quantize_layer_vq(np.array([[0.9, 0.1, 0.5, 0.5]]), np.eye(4), C)
    assert out["indices"].tolist() == [[0, 0]]              # (0.5, 0.5) is equidistant from entries 0 and 1
