"""Pins of the LoPRo pre-conditioning oracle (CPU only): what the paper and the mathematics fix."""
import numpy as np
import pytest
import scipy.linalg

from oracle import lopro_oracle as lo
from oracle import ptq_oracle as orc


def test_column_keys_hand_worked():
    # Eq. 5 on a 2 x 3 residual: amean = (|1|+|3|)/2, (|-2|+|2|)/2, (0+0)/2
    R = np.array([[1.0, -2.0, 0.0], [3.0, 2.0, 0.0]])
    H = np.diag([4.0, 6.0, 5.0]) + 0.5
    keys = lo.column_keys(H, R)
    assert keys[0] == 4.5 / 2.0 and keys[1] == 6.5 / 2.0 and np.isinf(keys[2])
    # a dead channel with a zero residual column ranks last in the default order, not first
    H[2, 2] = 0.0
    assert lo.column_keys(H, R)[2] == 0.0


def test_permutation_hand_worked_and_ties():
    keys = np.array([3.0, 7.0, 3.0, np.inf, 0.5])
    assert lo.permutation(keys).tolist() == [3, 1, 0, 2, 4]            # descending, ties by index
    assert lo.permutation(keys, descending=False).tolist() == [4, 0, 2, 1, 3]
    rng = np.random.default_rng(0)
    k = rng.standard_normal(500) ** 2
    p = lo.permutation(k)
    assert sorted(p.tolist()) == list(range(500))
    assert np.all(np.diff(k[p]) <= 0)


def test_permutation_matrix_is_a_gather():
    rng = np.random.default_rng(1)
    R = rng.standard_normal((3, 6))
    perm = np.array([4, 0, 5, 1, 3, 2])
    P = lo.permutation_matrix(perm)
    assert np.array_equal(R @ P, R[:, perm])
    assert np.array_equal(P.T @ P, np.eye(6))


@pytest.mark.parametrize("b", [1, 2, 8, 64, 256])
def test_hadamard_against_library_and_orthogonal(b):
    Hm = lo.hadamard(b)
    assert np.array_equal(Hm * np.sqrt(b), scipy.linalg.hadamard(b).astype(np.float64))
    assert np.allclose(Hm.T @ Hm, np.eye(b), atol=1e-14)
    assert np.array_equal(Hm, Hm.T)


def test_rotation_matrix_structure():
    Q = lo.rotation_matrix(24, 8, 4)
    assert np.array_equal(Q[:8, :8], np.eye(8))
    assert np.array_equal(Q[8:12, 8:12], lo.hadamard(4)) and np.array_equal(Q[20:, 20:], lo.hadamard(4))
    assert np.count_nonzero(Q) == 8 + 4 * 16
    assert np.allclose(Q.T @ Q, np.eye(24), atol=1e-15)
    with pytest.raises(AssertionError):
        lo.rotation_matrix(22, 8, 4)


def test_round_trip_is_exact_on_dyadic_inputs():
    # Q is orthogonal and symmetric with entries +-1/16 (b_H = 256) resp. +-1/4: integers survive exactly
    rng = np.random.default_rng(2)
    for n, bI, bH in [(1024, 256, 256), (48, 16, 16)]:
        R = rng.integers(-50, 50, size=(5, n)).astype(np.float64)
        perm = rng.permutation(n)
        Rr = lo.rotate_weight(R, perm, bI, bH)
        assert np.array_equal(Rr[:, :bI], R[:, perm[:bI]])                 # identity block: permuted only
        assert np.array_equal(lo.unrotate_weight(Rr, perm, bI, bH), R)
        assert np.allclose(np.linalg.norm(Rr, axis=1), np.linalg.norm(R, axis=1), rtol=1e-14)


def test_loss_invariance_and_decoupling():
    # Eq. 8 / Theorem 2: the loss of any quantized R' under H' equals the loss of its image under H,
    # and Eq. 7: R X = R' Q^T P^T X
    rng = np.random.default_rng(3)
    m, n, t, bI, bH = 6, 40, 90, 8, 16
    X = rng.standard_normal((t, n)) * np.exp(rng.standard_normal(n))
    H = orc.hessian(X)
    R = rng.standard_normal((m, n)) * 0.02
    perm = lo.permutation(lo.column_keys(H, R))
    Rr = lo.rotate_weight(R, perm, bI, bH)
    Hr = lo.rotate_hessian(H, perm, bI, bH)
    Rq = np.round(Rr * 64) / 64                                            # some quantization of R'
    back = lo.unrotate_weight(Rq, perm, bI, bH)
    loss_rot = np.trace((Rq - Rr) @ Hr @ (Rq - Rr).T)
    loss_orig = np.trace((back - R) @ H @ (back - R).T)
    assert abs(loss_rot - loss_orig) <= 1e-12 * loss_orig
    assert abs(loss_orig - np.linalg.norm((back - R) @ X.T) ** 2) <= 1e-10 * loss_orig
    Xt = (lo.rotation_matrix(n, bI, bH).T @ lo.permutation_matrix(perm).T @ X.T)   # activations as served
    assert np.allclose(R @ X.T, Rr @ Xt, rtol=1e-12, atol=1e-12)


def test_rotated_hessian_is_an_orthogonal_similarity():
    rng = np.random.default_rng(4)
    n, bI, bH = 64, 16, 16
    A = rng.standard_normal((200, n))
    H = A.T @ A
    perm = rng.permutation(n)
    Hr = lo.rotate_hessian(H, perm, bI, bH)
    assert np.allclose(Hr, Hr.T, atol=1e-12)
    assert abs(np.trace(Hr) - np.trace(H)) <= 1e-12 * np.trace(H)
    assert np.allclose(np.linalg.eigvalsh(Hr), np.linalg.eigvalsh(H), rtol=1e-10)
    assert np.allclose(Hr[:bI, :bI], H[np.ix_(perm[:bI], perm[:bI])], atol=0)    # identity block: a pure gather
    # entry-wise: H'[a, b] = sum_ij Q[i, a] Hp[i, j] Q[j, b]
    Q = lo.rotation_matrix(n, bI, bH)
    Hp = H[np.ix_(perm, perm)]
    a, b = 20, 37
    ref = sum(Q[i, a] * Hp[i, j] * Q[j, b] for i in range(n) for j in range(n))
    assert abs(Hr[a, b] - ref) <= 1e-10 * abs(ref)


def test_solve_in_rotated_basis_is_a_valid_solve():
    # the unchanged column solve applied to (R', H') and mapped back reproduces its own loss (sum e^2
    # identity of the solve, with the damped rotated Hessian)
    rng = np.random.default_rng(5)
    m, n, t, bI, bH = 8, 64, 300, 16, 16
    X = rng.standard_normal((t, n)) @ (np.eye(n) + 0.5 * rng.standard_normal((n, n)) / np.sqrt(n))
    H = orc.hessian(X)
    R = rng.standard_normal((m, n)) * 0.02
    perm = lo.permutation(lo.column_keys(H, R))
    Rr, Hr = lo.rotate_weight(R, perm, bI, bH), lo.rotate_hessian(H, perm, bI, bH)
    Hd, dead = orc.damp(Hr, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    out = orc.quantize_layer(Rr, U, 4, 16, dead=dead)
    back = lo.unrotate_weight(out["Wq"], perm, bI, bH)
    e_rot = orc.layer_error(Rr, out["Wq"], Hr)[0]
    e_orig = orc.layer_error(R, back, H)[0]
    assert abs(e_rot - e_orig) <= 1e-10
