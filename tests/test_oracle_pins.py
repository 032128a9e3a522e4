"""Pins for the CPU oracle: each test checks it against something that is not
itself -- closed forms worked by hand, brute force, least-squares optimality,
identities that follow from the objective (Sec. 2, Eq. 1 of the paper).  They
are chosen so that a dropped term, a wrong sign or index, or a transposed
operand in the oracle fails at least one of them."""
import itertools
import math

import numpy as np
import pytest

from oracle import ptq_oracle as orc


def _spd(n, rng, corr=0.9, t=None):
    """A strongly correlated Hessian X^T X (so that compensation matters)."""
    t = t or 3 * n
    A = rng.standard_normal((n, n))
    Z = rng.standard_normal((t, n))
    X = Z @ (np.eye(n) + corr * A / math.sqrt(n))
    X *= np.exp(rng.standard_normal(n))
    return X.T @ X, X


# ------------------------------------------------------------------ Hessian
def test_hessian_brute_force():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((37, 5))
    H = orc.hessian(X, chunk=8)
    for i in range(5):
        for j in range(5):
            s = 0.0
            for t in range(37):
                s += X[t, i] * X[t, j]
            assert abs(H[i, j] - s) < 1e-12


def test_hessian_closed_forms_and_accumulation():
    t, n = 50, 7
    H = orc.hessian(np.ones((t, n)))
    assert np.array_equal(H, t * np.ones((n, n)))
    # one-hot tokens: token k fires channel k % n with amplitude k+1
    X = np.zeros((t, n))
    for k in range(t):
        X[k, k % n] = k + 1
    H = orc.hessian(X)
    expect = np.diag([sum((k + 1) ** 2 for k in range(t) if k % n == c) for c in range(n)])
    assert np.array_equal(H, expect)
    # accumulating two slabs equals one pass
    rng = np.random.default_rng(2)
    X = rng.standard_normal((64, 6))
    H2 = orc.hessian(X[:40])
    H2 = orc.hessian(X[40:], H2)
    assert np.allclose(H2, orc.hessian(X), rtol=0, atol=1e-12)
    # a transposed operand would give a 64x64 matrix
    assert H2.shape == (6, 6)


# ------------------------------------------------------------- damp + factor
def test_damp_closed_form():
    H = np.array([[2.0, 1.0, 0.0], [1.0, 4.0, 0.0], [0.0, 0.0, 0.0]])
    Hd, dead = orc.damp(H, 0.5)
    assert dead.tolist() == [False, False, True]
    mean = (2.0 + 4.0 + 1.0) / 3.0
    expect = np.array([[2.0, 1.0, 0.0], [1.0, 4.0, 0.0], [0.0, 0.0, 1.0]]) + 0.5 * mean * np.eye(3)
    assert np.allclose(Hd, expect, rtol=0, atol=1e-15)
    assert np.array_equal(H, np.array([[2.0, 1.0, 0.0], [1.0, 4.0, 0.0], [0.0, 0.0, 0.0]]))


def test_factor_hand_worked_2x2():
    # H = [[4,2],[2,3]], H^-1 = 1/8 [[3,-2],[-2,4]];  U^T U = H^-1, U upper:
    # U11^2 = 3/8, U11 U12 = -1/4, U12^2 + U22^2 = 1/2.
    U = orc.inverse_cholesky_upper(np.array([[4.0, 2.0], [2.0, 3.0]]))
    u11 = math.sqrt(3.0 / 8.0)
    u12 = -0.25 / u11
    u22 = math.sqrt(0.5 - u12 * u12)
    assert np.allclose(U, [[u11, u12], [0.0, u22]], rtol=0, atol=1e-15)
    assert abs(u22 - 1 / math.sqrt(3.0)) < 1e-15


def test_factor_hand_worked_3x3():
    # H = R R^T with R upper, built from the last row upwards by hand; U = R^-1.
    H = np.array([[4.0, 2.0, 0.0], [2.0, 5.0, 1.0], [0.0, 1.0, 3.0]])
    r33 = math.sqrt(3.0)
    r23 = 1.0 / r33
    r13 = 0.0
    r22 = math.sqrt(5.0 - r23 ** 2)
    r12 = (2.0 - r13 * r23) / r22
    r11 = math.sqrt(4.0 - r12 ** 2 - r13 ** 2)
    u = np.array([[1 / r11, -r12 / (r11 * r22), (r12 * r23 - r13 * r22) / (r11 * r22 * r33)],
                  [0.0, 1 / r22, -r23 / (r22 * r33)],
                  [0.0, 0.0, 1 / r33]])
    U = orc.inverse_cholesky_upper(H)
    assert np.allclose(U, u, rtol=0, atol=1e-14)


@pytest.mark.parametrize("n", [1, 5, 64, 200])
def test_factor_properties_and_reversed_route(n):
    rng = np.random.default_rng(n)
    H, _ = _spd(n, rng)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    assert np.all(np.tril(U, -1) == 0) and np.all(np.diag(U) > 0)
    assert np.allclose(U.T @ U @ Hd, np.eye(n), rtol=0, atol=1e-8)
    # uniqueness: Cholesky of the index-reversed matrix, reversed back and
    # inverted, is the same factor.
    J = np.arange(n)[::-1]
    Lr = np.linalg.cholesky(Hd[np.ix_(J, J)])
    R = Lr[np.ix_(J, J)]
    assert np.allclose(R @ R.T, Hd, rtol=0, atol=1e-12 * np.abs(Hd).max())
    U2 = np.linalg.inv(R)
    scale = np.abs(U).max()
    assert np.allclose(U, U2, rtol=0, atol=1e-9 * scale)


# ------------------------------------------------------------- quantize_layer
def _on_grid_layer(rng, m, n, group, bits, pow2=True):
    maxq = 2 ** bits - 1
    codes = rng.integers(0, maxq + 1, size=(m, n))
    ng = n // group
    scales = 2.0 ** rng.integers(-8, -2, size=(m, ng)) if pow2 else \
        rng.uniform(0.01, 0.1, size=(m, ng)).astype(np.float32).astype(np.float64)
    zeros = rng.integers(1, maxq, size=(m, ng))
    for r in range(m):                       # every group holds code 0 and maxq
        for k in range(ng):
            a, b = rng.choice(group, 2, replace=False)
            codes[r, k * group + a] = 0
            codes[r, k * group + b] = maxq
    W = np.repeat(scales, group, axis=1) * (codes - np.repeat(zeros, group, axis=1))
    return W, codes, scales, zeros


@pytest.mark.parametrize("bits,group", [(2, 8), (3, 16), (4, 32), (8, 32)])
def test_on_grid_recovery(bits, group):
    rng = np.random.default_rng(bits * 100 + group)
    m, n = 6, 64
    W, codes, scales, zeros = _on_grid_layer(rng, m, n, group, bits)
    H, _ = _spd(n, rng)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    out = orc.quantize_layer(W, U, bits, group)
    assert np.array_equal(out["codes"], codes)
    assert np.array_equal(out["scales"].astype(np.float64), scales)
    assert np.array_equal(out["zeros"], zeros)
    assert np.all(out["E"] == 0) and np.array_equal(out["Wq"], W)
    rel, num, den = orc.layer_error(W, out["Wq"], H)
    assert rel == 0.0 and num == 0.0 and den > 0


def test_diagonal_hessian_is_round_to_nearest():
    rng = np.random.default_rng(7)
    m, n, group, bits = 9, 96, 32, 3
    W = rng.standard_normal((m, n)) * 0.02
    W[:, 5] *= 10
    Hd = np.diag(rng.uniform(0.5, 50.0, n))
    U = orc.inverse_cholesky_upper(Hd)
    assert np.allclose(U, np.diag(1 / np.sqrt(np.diag(Hd))), rtol=1e-13, atol=0)
    out = orc.quantize_layer(W, U, bits, group)
    # textbook round-to-nearest written out with python scalars
    maxq = 2 ** bits - 1
    for r in range(m):
        for k in range(n // group):
            g = W[r, k * group:(k + 1) * group]
            lo, hi = min(0.0, g.min()), max(0.0, g.max())
            s = float(np.float32((hi - lo) / maxq))
            z = round(-lo / s)               # python round is half-to-even
            assert out["scales"][r, k] == np.float32(s) and out["zeros"][r, k] == z
            for i, w in enumerate(g):
                c = min(max(round(w / s) + z, 0), maxq)
                assert out["codes"][r, k * group + i] == c
    rtn = orc.round_to_nearest(W, bits, group)
    assert np.array_equal(rtn["codes"], out["codes"])


def test_degenerate_group_and_dead_column():
    n, group, bits = 16, 8, 4
    W = np.zeros((2, n))
    W[1, 8:] = np.linspace(-0.3, 0.4, 8)
    W[:, 3] = 5.0                                   # lives in a dead channel
    dead = np.zeros(n, dtype=bool)
    dead[3] = True
    U = np.eye(n)
    out = orc.quantize_layer(W, U, bits, group, dead=dead)
    # all-zero group: range [-1, 1]; float32(2/15) lies above 2/15, so
    # 1/scale is just below 7.5 and the zero-point is 7; code 7 -> q = 0
    assert out["scales"][0, 0] == np.float32(2.0 / 15.0)
    assert float(np.float32(2.0 / 15.0)) > 2.0 / 15.0
    assert out["zeros"][0, 0] == 7 and np.all(out["codes"][0] == 7)
    assert np.all(out["Wq"][0] == 0.0) and out["Wq"][1, 3] == 0.0


def _schur_loss(Hd, d_head):
    """min over the free tail of d^T Hd d with the head of d fixed."""
    j = len(d_head)
    n = Hd.shape[0]
    if j == n:
        return float(d_head @ Hd @ d_head)
    Haa, Hab, Hbb = Hd[:j, :j], Hd[:j, j:], Hd[j:, j:]
    S = Haa - Hab @ np.linalg.solve(Hbb, Hab.T)
    return float(d_head @ S @ d_head)


@pytest.mark.parametrize("seed", range(6))
def test_conditional_optimality(seed):
    """Each code minimises the damped loss over its own column, given the
    earlier codes, when the later columns are left continuous and optimal.
    The check uses only H_d (a Schur complement), never U."""
    rng = np.random.default_rng(100 + seed)
    n, bits, group = 6, 3, 3
    maxq = 2 ** bits - 1
    H, _ = _spd(n, rng)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    W = rng.standard_normal((4, n)) * 0.05
    out = orc.quantize_layer(W, U, bits, group)
    for r in range(W.shape[0]):
        for j in range(n):
            s = float(out["scales"][r, j // group])
            z = float(out["zeros"][r, j // group])
            head = W[r, :j] - out["Wq"][r, :j]
            losses = [_schur_loss(Hd, np.append(head, W[r, j] - s * (c - z)))
                      for c in range(maxq + 1)]
            best = int(np.argmin(losses))
            chosen = int(out["codes"][r, j])
            assert losses[chosen] <= losses[best] * (1 + 1e-9) + 1e-18, (r, j, chosen, best)


@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_brute_force_small(n):
    rng = np.random.default_rng(40 + n)
    bits, group = 2, n
    maxq = 3
    worse = 0
    for trial in range(20):
        H, _ = _spd(n, rng, t=n + 2)
        Hd, _ = orc.damp(H, 0.01)
        U = orc.inverse_cholesky_upper(Hd)
        W = rng.standard_normal((1, n)) * 0.1
        out = orc.quantize_layer(W, U, bits, group)
        s = float(out["scales"][0, 0])
        z = float(out["zeros"][0, 0])
        d = W[0] - out["Wq"][0]
        got = float(d @ Hd @ d)
        best = min(float((W[0] - s * (np.array(c) - z)) @ Hd @ (W[0] - s * (np.array(c) - z)))
                   for c in itertools.product(range(maxq + 1), repeat=n))
        assert best <= got * (1 + 1e-12) + 1e-18
        if n == 1:
            assert abs(best - got) <= 1e-12 * got + 1e-18
        # the greedy result is also never worse than plain rounding here
        rtn = orc.round_to_nearest(W, bits, group)
        dr = W[0] - rtn["Wq"][0]
        worse += float(dr @ Hd @ dr) < got * (1 - 1e-12)
    assert worse <= 2


@pytest.mark.parametrize("seed", range(4))
def test_error_identity(seed):
    """(W - Wq) = E U row-wise, hence tr(D H_d D^T) = sum e^2."""
    rng = np.random.default_rng(200 + seed)
    m, n, bits, group = 5, 48, 4, 16
    H, _ = _spd(n, rng)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    W = rng.standard_normal((m, n)) * 0.02
    out = orc.quantize_layer(W, U, bits, group)
    D = W - out["Wq"]
    assert np.allclose(D, out["E"] @ U, rtol=0, atol=1e-12 * np.abs(W).max())
    lhs = np.einsum("ij,ij->i", D @ Hd, D)
    assert np.allclose(lhs, out["row_err2"], rtol=1e-9, atol=0)
    assert np.allclose(out["Wq"], orc.dequantize(out["codes"], out["scales"], out["zeros"], group))
    # codes do not depend on a positive rescale of H (damping is relative)
    Hd2, _ = orc.damp(7.5 * H, 0.01)
    out2 = orc.quantize_layer(W, orc.inverse_cholesky_upper(Hd2), bits, group)
    assert np.array_equal(out["codes"], out2["codes"])


def test_not_worse_than_rtn_on_correlated_layers():
    wins = 0
    total = 12
    for seed in range(total):
        rng = np.random.default_rng(300 + seed)
        m, n, bits, group = 16, 64, 3, 32
        H, X = _spd(n, rng, t=80)
        Hd, dead = orc.damp(H, 0.01)
        U = orc.inverse_cholesky_upper(Hd)
        W = rng.standard_normal((m, n)) * 0.02
        a = orc.layer_error(W, orc.quantize_layer(W, U, bits, group)["Wq"], H)[0]
        b = orc.layer_error(W, orc.round_to_nearest(W, bits, group)["Wq"], H)[0]
        wins += a <= b
    assert wins == total


def test_forced_decisions_are_applied():
    rng = np.random.default_rng(5)
    n, bits, group = 32, 4, 16
    H, _ = _spd(n, rng)
    U = orc.inverse_cholesky_upper(orc.damp(H, 0.01)[0])
    W = rng.standard_normal((3, n)) * 0.02
    base = orc.quantize_layer(W, U, bits, group, want_pre=True)
    c = int(base["codes"][1, 5])
    alt = c + 1 if c < 15 else c - 1
    out = orc.quantize_layer(W, U, bits, group, forced={("code", 1, 5): alt})
    assert out["codes"][1, 5] == alt
    assert np.array_equal(out["codes"][[0, 2]], base["codes"][[0, 2]])
    assert np.array_equal(out["codes"][1, :5], base["codes"][1, :5])
    z = int(base["zeros"][2, 1])
    out = orc.quantize_layer(W, U, bits, group, forced={("zero", 2, 1): z + 1})
    assert out["zeros"][2, 1] == z + 1 and np.array_equal(out["codes"][2, :16], base["codes"][2, :16])


# ------------------------------------------------------------- layer error
def test_trace_identity_and_permutation_covariance():
    rng = np.random.default_rng(11)
    m, n = 7, 24
    H, X = _spd(n, rng)
    W = rng.standard_normal((m, n))
    Wq = W + 0.05 * rng.standard_normal((m, n))
    rel, num, den = orc.layer_error(W, Wq, H)
    assert abs(rel - orc.layer_error_from_activations(W, Wq, X)) < 1e-12
    # num is a plain quadratic form
    D = W - Wq
    s = sum(D[r, i] * H[i, j] * D[r, j] for r in range(m) for i in range(n) for j in range(n))
    assert abs(num - s) < 1e-9 * abs(s)
    # the loss is the same in a permuted / rotated basis (Sec. 3.2, Eq. 8)
    Q, _ = np.linalg.qr(rng.standard_normal((n, n)))
    rel2 = orc.layer_error(W @ Q, Wq @ Q, Q.T @ H @ Q)[0]
    assert abs(rel - rel2) < 1e-10
    p = rng.permutation(n)
    rel3 = orc.layer_error(W[:, p], Wq[:, p], H[np.ix_(p, p)])[0]
    assert abs(rel - rel3) < 1e-12
    Hu = np.triu(H) + 123.0 * np.tril(np.ones((n, n)), -1)
    assert np.array_equal(orc.symmetrize_from_upper(Hu), np.triu(H) + np.triu(H, 1).T)


# ---------------------------------------------------------- static groups
def test_static_groups_grids_are_those_of_the_given_weights():
    """With static groups every scale and zero is the round-to-nearest grid of the weights as handed
    over: independent of the Hessian, and equal to the textbook min / max grid written out by hand."""
    rng = np.random.default_rng(410)
    m, n, bits, group = 6, 64, 3, 16
    W = rng.standard_normal((m, n)) * 0.02
    W[:, 3] *= 12
    maxq = 2 ** bits - 1
    outs = []
    for seed in (1, 2):
        H, _ = _spd(n, np.random.default_rng(seed))
        Hd, _ = orc.damp(H, 0.01)
        outs.append(orc.quantize_layer(W, orc.inverse_cholesky_upper(Hd), bits, group, static_groups=True))
    assert np.array_equal(outs[0]["scales"], outs[1]["scales"]) and np.array_equal(outs[0]["zeros"], outs[1]["zeros"])
    assert not np.array_equal(outs[0]["codes"], outs[1]["codes"])      # the codes do feel the Hessian
    for r in range(m):
        for k in range(n // group):
            g = W[r, k * group:(k + 1) * group]
            lo, hi = min(0.0, g.min()), max(0.0, g.max())
            s = float(np.float32((hi - lo) / maxq))
            assert outs[0]["scales"][r, k] == np.float32(s) and outs[0]["zeros"][r, k] == round(-lo / s)
    # the grids of the ordinary solve move with the compensation (first group aside)
    dyn = orc.quantize_layer(W, orc.inverse_cholesky_upper(orc.damp(_spd(n, np.random.default_rng(1))[0], 0.01)[0]),
                             bits, group)
    assert np.array_equal(dyn["scales"][:, 0], outs[0]["scales"][:, 0])
    assert not np.array_equal(dyn["scales"][:, 1:], outs[0]["scales"][:, 1:])


def test_static_groups_keep_the_identities_of_the_solve():
    """Where the grid comes from does not touch the compensation: (W - Wq) = E U and sum e^2 =
    tr(D H_d D^T) still hold, a diagonal Hessian still gives round-to-nearest, and weights on the grid
    are still recovered exactly."""
    rng = np.random.default_rng(411)
    m, n, bits, group = 5, 48, 4, 16
    H, _ = _spd(n, rng)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    W = rng.standard_normal((m, n)) * 0.02
    out = orc.quantize_layer(W, U, bits, group, static_groups=True)
    D = W - out["Wq"]
    assert np.allclose(D, out["E"] @ U, rtol=0, atol=1e-12 * np.abs(W).max())
    assert np.allclose(np.einsum("ij,ij->i", D @ Hd, D), out["row_err2"], rtol=1e-9, atol=0)
    assert np.allclose(out["Wq"], orc.dequantize(out["codes"], out["scales"], out["zeros"], group))
    Udiag = orc.inverse_cholesky_upper(np.diag(rng.uniform(0.5, 50.0, n)))
    a = orc.quantize_layer(W, Udiag, bits, group, static_groups=True)
    b = orc.quantize_layer(W, Udiag, bits, group)
    assert all(np.array_equal(a[k], b[k]) for k in ("codes", "scales", "zeros"))
    rtn = orc.round_to_nearest(W, bits, group)
    on_grid = orc.dequantize(rtn["codes"], rtn["scales"], rtn["zeros"], group)
    c = orc.quantize_layer(on_grid, U, bits, group, static_groups=True)
    assert np.array_equal(c["Wq"], on_grid)


def test_dynamic_grid_is_taken_when_the_walk_enters_the_group_hand_worked():
    """Pins WHEN a group's grid is taken: from the row's values after every earlier column's error
    has been pushed onto them and before the group's own first column is quantized.  Worked by hand:
    2 bits (codes 0..3), groups of 2, four columns, U = I except U[1,3] = 4 (the last column of the
    first group pushes onto the second group) and U[2,3] = 8 (the second group's first column pushes
    onto its second).

    row 0: w = (3, 1.25, 1.5, 7)
      group 0: range [0, 3], scale 1, zero 0.  col 0: code 3, e = 0.  col 1: 1.25 -> code 1, q = 1,
               e = 0.25, so w3 = 7 - 0.25 * 4 = 6.
      group 1, taken now: values (1.5, 6) -> range [0, 6], scale 2, zero 0.
               col 2: 0.75 -> code 1, q = 2, e = -0.5, so w3 = 6 + 0.5 * 8 = 10.
               col 3: 10 / 2 = 5 -> clamped to code 3, q = 6, e = 4.
      (from the weights as given the scale would be 7/3; taken one column later, after col 2's
       push, 10/3.)
    row 1: w = (-3, -1.25, -0.5, -7)
      group 0: range [-3, 0], scale 1, zero 3.  col 0: code 0, e = 0.  col 1: -1.25 -> -1 + 3 = 2,
               q = -1, e = -0.25, so w3 = -7 + 0.25 * 4 = -6.
      group 1, taken now: values (-0.5, -6) -> range [-6, 0], scale 2, zero 3.
               col 2: -0.25 -> rounds to -0 -> code 3, q = 0, e = -0.5, so w3 = -6 + 0.5 * 8 = -2.
               col 3: -2 / 2 = -1 -> code 2, q = -2, e = 0.
    """
    W = np.array([[3.0, 1.25, 1.5, 7.0], [-3.0, -1.25, -0.5, -7.0]])
    U = np.eye(4)
    U[1, 3] = 4.0
    U[2, 3] = 8.0
    out = orc.quantize_layer(W, U, 2, 2)
    assert out["scales"].tolist() == [[1.0, 2.0], [1.0, 2.0]]
    assert out["zeros"].tolist() == [[0, 0], [3, 3]]
    assert out["codes"].tolist() == [[3, 1, 1, 3], [0, 2, 3, 2]]
    assert out["Wq"].tolist() == [[3.0, 1.0, 2.0, 6.0], [-3.0, -1.0, 0.0, -2.0]]
    assert out["E"].tolist() == [[0.0, 0.25, -0.5, 4.0], [0.0, -0.25, -0.5, 0.0]]
    # the static-groups option is the other timing: grids of the weights as given
    st = orc.quantize_layer(W, U, 2, 2, static_groups=True)
    assert st["scales"][:, 1].tolist() == [float(np.float32(7.0 / 3.0))] * 2
