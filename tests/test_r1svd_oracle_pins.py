"""Pins for oracle/r1svd_oracle.py: every function is held against something that is not
itself -- torch's float8 conversion, hand-worked numbers, closed forms of Eq. 9-11,
numpy's SVD, the Eckart-Young bound."""
import numpy as np
import pytest
import torch

from oracle import r1svd_oracle as ro


# ---------------------------------------------------------------- e4m3 ----------------
def _torch_e4m3(x):
    t = torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy(), t.to(torch.float32).numpy().astype(np.float64)


def test_e4m3_code_table_matches_torch():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = ro.e4m3_decode(codes)
    assert np.array_equal(got, want.astype(np.float64))
    assert np.array_equal(np.signbit(got), np.signbit(want))
    # and back
    val, _ = ro.e4m3_round(got)
    assert np.array_equal(ro.e4m3_encode(val), codes)


def test_e4m3_rounding_matches_torch_on_float32_values():
    rng = np.random.default_rng(5)
    x = np.concatenate([
        rng.standard_normal(20000) * 0.02,           # the range unit vectors of length ~4096 live in
        rng.standard_normal(20000),
        rng.uniform(-0.004, 0.004, 5000),            # subnormals and flush to zero
        rng.uniform(-464, 464, 2000),                # up to the last value that rounds to 448
        np.array([0.0, -0.0, 2.0 ** -10, -2.0 ** -10, 3 * 2.0 ** -10, 448.0, 464.0]),
    ]).astype(np.float32)
    # every exact tie between neighbouring codes as well
    tab = np.sort(ro.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8)))
    ties = (tab[1:] + tab[:-1]) / 2
    x = np.concatenate([x, ties.astype(np.float32), -ties.astype(np.float32)])
    assert np.array_equal(ties, ties.astype(np.float32).astype(np.float64))
    want_code, want_val = _torch_e4m3(x)
    val, margin = ro.e4m3_round(x.astype(np.float64))
    assert np.array_equal(val, want_val)
    assert np.array_equal(ro.e4m3_encode(val), want_code)
    k = x.size - 2 * ties.size
    assert np.all(margin[k:] == 0.0)
    assert np.all((margin >= 0) & (margin <= 0.5))
    # beyond that torch's conversion gives NaN; the oracle saturates (never reached by the
    # method: it only converts entries of unit vectors)
    assert np.array_equal(ro.e4m3_round(np.array([1e6, -465.0]))[0], [448.0, -448.0])


def test_e4m3_margin_is_distance_to_tie_in_quanta():
    # 0.3 lies in [0.25, 0.5): quantum 1/32; 0.3 * 32 = 9.6 -> frac 0.6 -> 0.1 from the tie
    _, mg = ro.e4m3_round(np.array([0.3]))
    assert mg[0] == pytest.approx(0.1, abs=1e-12)


# ---------------------------------------------------------------- scale ----------------
def test_scale_hand_worked():
    # Xbar = (1, 4, 16): max*min = 16, sqrt = 4; Xbar^2.5 = (1, 32, 1024)
    X = np.array([[1.0, -4.0, 16.0], [-1.0, 4.0, -16.0]])
    xbar = ro.mean_abs_activation(X)
    assert np.array_equal(xbar, [1.0, 4.0, 16.0])
    assert np.allclose(ro.activation_scale(xbar), [0.25, 8.0, 256.0], rtol=1e-15)


def test_scale_closed_forms():
    # constant Xbar = c  ->  s = c^1.5 ; scaling X by a scales s by a^1.5
    assert np.allclose(ro.activation_scale(np.full(7, 2.25)), 2.25 ** 1.5)
    rng = np.random.default_rng(3)
    xb = rng.uniform(0.1, 5, 50)
    assert np.allclose(ro.activation_scale(3.0 * xb), 3.0 ** 1.5 * ro.activation_scale(xb), rtol=1e-13)
    # the geometric mean of s at the extreme channels: s_max * s_min = (max*min)^1.5
    s = ro.activation_scale(xb)
    assert s[np.argmax(xb)] * s[np.argmin(xb)] == pytest.approx((xb.max() * xb.min()) ** 1.5, rel=1e-13)


def test_scale_dead_channel_reading():
    s = ro.activation_scale(np.array([0.0, 1.0, 4.0]))
    assert np.allclose(s, [1.0, 0.5, 16.0])
    assert np.all(ro.activation_scale(np.zeros(4)) == 1.0)


# ---------------------------------------------------------------- one step -------------
def test_rank_one_matrix_is_recovered_exactly():
    rng = np.random.default_rng(11)
    a = rng.standard_normal(40)
    b = rng.standard_normal(30)
    A = np.outer(a, b)
    v = rng.standard_normal(30)
    for it in (0, 1, 3):
        u, sg, vv = ro.rank_one_step(A, v, it)
        sign = np.sign(u @ a)
        assert np.allclose(u, sign * a / np.linalg.norm(a), atol=1e-13)
        assert np.allclose(vv, sign * b / np.linalg.norm(b), atol=1e-13)
        assert sg == pytest.approx(np.linalg.norm(a) * np.linalg.norm(b), rel=1e-13)


def test_step_is_the_printed_formula_with_an_explicit_matrix_power():
    rng = np.random.default_rng(12)
    A = rng.standard_normal((12, 9))
    v = rng.standard_normal(9)
    it = 3
    y = np.linalg.matrix_power(A @ A.T, it) @ A @ v
    p = v @ A.T @ np.linalg.matrix_power(A @ A.T, it) @ A        # S* A* (A A*)^it A, Eq. 11
    u, sg, vv = ro.rank_one_step(A, v, it)
    assert np.allclose(u, y / np.linalg.norm(y), rtol=1e-12, atol=1e-14)
    assert np.allclose(vv, p / np.linalg.norm(p), rtol=1e-12, atol=1e-14)
    assert sg == pytest.approx(np.linalg.norm(p) / np.linalg.norm(y), rel=1e-12)


def test_step_converges_to_the_leading_singular_triplet():
    rng = np.random.default_rng(13)
    m, n = 60, 45
    Uo, _ = np.linalg.qr(rng.standard_normal((m, m)))
    Vo, _ = np.linalg.qr(rng.standard_normal((n, n)))
    sv = np.concatenate([[10.0, 4.0], np.linspace(2.0, 0.1, n - 2)])
    A = (Uo[:, :n] * sv) @ Vo.T
    u, sg, vv = ro.rank_one_step(A, rng.standard_normal(n), 8)
    Ul, sl, Vlt = np.linalg.svd(A)
    assert sg == pytest.approx(sl[0], rel=1e-6)          # (4/10)^(2*8+1) contamination at most
    assert abs(u @ Ul[:, 0]) == pytest.approx(1.0, abs=1e-6)
    assert abs(vv @ Vlt[0]) == pytest.approx(1.0, abs=1e-6)
    assert (u @ Ul[:, 0]) * (vv @ Vlt[0]) > 0            # u sigma v^T has the right sign
    # sigma never exceeds the largest singular value, whatever the iteration count
    for it in (0, 1, 2):
        assert ro.rank_one_step(A, rng.standard_normal(n), it)[1] <= sl[0] * (1 + 1e-12)


def test_zero_matrix_gives_zero_factors():
    u, sg, vv = ro.rank_one_step(np.zeros((5, 4)), np.ones(4), 2)
    assert sg == 0.0 and not u.any() and not vv.any()


# ---------------------------------------------------------------- the loop -------------
def _gapped(rng, m, n, lead):
    Uo, _ = np.linalg.qr(rng.standard_normal((m, m)))
    Vo, _ = np.linalg.qr(rng.standard_normal((n, n)))
    k = min(m, n)
    sv = np.concatenate([lead, np.linspace(1.0, 0.2, k - len(lead))])
    return (Uo[:, :k] * sv) @ Vo[:, :k].T, sv


def test_unrounded_loop_approaches_eckart_young_and_never_beats_it():
    rng = np.random.default_rng(21)
    A, sv = _gapped(rng, 70, 50, np.array([40.0, 25.0, 16.0, 9.0]))
    S = rng.standard_normal((4, 50))
    out = ro.r1svd(A, S, 8, rounded=False)
    best = np.sqrt(np.sum(sv[4:] ** 2))
    err = np.linalg.norm(out["A"])
    assert err >= best * (1 - 1e-12)
    assert err <= best * 1.01
    assert np.allclose(out["sigma"], sv[:4], rtol=1e-3)
    # with few iterations and no gap the bound still holds
    B = rng.standard_normal((30, 20))
    o2 = ro.r1svd(B, rng.standard_normal((5, 20)), 1, rounded=False)
    sb = np.linalg.svd(B, compute_uv=False)
    assert np.linalg.norm(o2["A"]) >= np.sqrt(np.sum(sb[5:] ** 2)) * (1 - 1e-12)


def test_unrounded_deflation_leaves_residual_orthogonal_to_each_found_pair():
    # A - sigma u v^T with v = A^T u / sigma: the deflated matrix satisfies u^T A' = 0, and
    # later ranks (built from A') keep their U orthogonal to the earlier ones
    rng = np.random.default_rng(22)
    A = rng.standard_normal((25, 18))
    out = ro.r1svd(A, rng.standard_normal((3, 18)), 2, rounded=False)
    G = out["U"] @ out["U"].T
    assert np.allclose(G, np.eye(3), atol=1e-12)
    assert np.allclose(out["U"] @ out["A"], 0.0, atol=1e-12)


def test_rounded_loop_reconstruction_identity_and_stored_formats():
    rng = np.random.default_rng(23)
    m, n, r = 48, 64, 6
    W, _ = _gapped(rng, m, n, np.array([30.0, 20.0, 12.0]))
    s = rng.uniform(0.2, 4.0, n)
    S = rng.standard_normal((r, n))
    out = ro.scaled_r1svd(W, s, S, 4)
    # what is stored reconstructs W exactly (up to fp64 rounding): W = W_r + R   (Eq. 4)
    assert np.allclose(ro.low_rank_weight(out, s) + out["R"], W, rtol=0, atol=1e-12 * np.abs(W).max())
    # stored values are e4m3 / fp16 numbers and the codes decode to them
    assert np.array_equal(ro.e4m3_decode(out["U_code"]), out["U"])
    assert np.array_equal(ro.e4m3_decode(out["V_code"]), out["V"])
    assert np.array_equal(out["sigma"], out["sigma"].astype(np.float16).astype(np.float64))
    assert np.all(np.abs(out["U"]) <= 1.0) and np.all(np.abs(out["V"]) <= 1.0)
    # rounding costs accuracy but the later ranks still reduce the error monotonically
    errs = [np.linalg.norm(ro.scaled_r1svd(W, s, S[:k], 4)["A"]) for k in range(1, r + 1)]
    assert all(b < a for a, b in zip(errs, errs[1:]))
    # and the scaled residual is much smaller than the scaled weight
    assert errs[2] < 0.5 * np.linalg.norm(W * s)


def test_rounded_differs_from_unrounded_only_by_the_rounding():
    rng = np.random.default_rng(24)
    A, _ = _gapped(rng, 32, 32, np.array([9.0]))
    S = rng.standard_normal((1, 32))
    a = ro.r1svd(A, S, 6, rounded=False)
    b = ro.r1svd(A, S, 6, rounded=True)
    want_u, _ = ro.e4m3_round(a["U"][0])
    assert np.array_equal(b["U"][0], want_u)
    assert b["sigma"][0] == float(np.float16(a["sigma"][0]))
    assert np.allclose(b["A"], A - b["sigma"][0] * np.outer(b["U"][0], b["V"][0]), atol=1e-14)


def test_forced_codes_replace_single_entries():
    rng = np.random.default_rng(25)
    A = rng.standard_normal((16, 12))
    S = rng.standard_normal((2, 12))
    base = ro.r1svd(A, S, 2)
    Uf = np.full((2, 16), -1, dtype=np.int16)
    Uf[0, 3] = int(base["U_code"][0, 3]) ^ 1
    forced = ro.r1svd(A, S, 2, U_force=Uf)
    assert forced["U_code"][0, 3] == Uf[0, 3]
    same = np.ones(16, bool); same[3] = False
    assert np.array_equal(forced["U_code"][0][same], base["U_code"][0][same])
    assert not np.array_equal(forced["A"], base["A"])
    none = ro.r1svd(A, S, 2, U_force=np.full((2, 16), -1, dtype=np.int16))
    assert np.array_equal(none["A"], base["A"])


def test_follow_protocol_adopts_only_legitimate_roundings():
    """The near-tie rule of the parity protocol (tests/parity.py), exercised on the CPU with a made-up
    'other implementation': the oracle's own results with one code moved to its neighbour."""
    from parity import follow_r1svd
    rng = np.random.default_rng(26)
    A = rng.standard_normal((16, 12))
    S = rng.standard_normal((2, 12))
    one = np.ones(12)
    base = ro.r1svd(A, S, 2)
    exact = ro.r1svd(A, S, 2, rounded=False)
    assert np.array_equal(base["U_exact"][0], exact["U"][0])      # rank 0 sees the same matrix either way
    # the other neighbour of the entry closest to a tie is adopted with a tolerance above its
    # margin, and refused with a tolerance below it; a far-off code is never adopted
    i = int(np.argmin(base["U_margin"][0]))
    mg = base["U_margin"][0, i]
    x = exact["U"][0, i]
    own = base["U"][0, i]
    q = 2.0 ** (max(np.frexp(abs(x))[1] - 1, -6) - 3)
    other = own + q if x > own else own - q
    theirs = {"U_code": base["U_code"].copy(), "V_code": base["V_code"].copy(), "sigma": base["sigma"].copy()}
    theirs["U_code"][0, i] = ro.e4m3_encode(np.array([other]))[0]
    yes = follow_r1svd(A, one, S, 2, theirs["U_code"], theirs["V_code"], theirs["sigma"], mg * 1.01 + 1e-12)
    assert yes["followed"] >= 1 and yes["U_code"][0, i] == theirs["U_code"][0, i]
    no = follow_r1svd(A, one, S, 2, theirs["U_code"], theirs["V_code"], theirs["sigma"], mg * 0.5)
    assert no["U_code"][0, i] == base["U_code"][0, i] and no["followed"] == 0
    far = {k: v.copy() for k, v in theirs.items()}
    far["U_code"][0, i] = base["U_code"][0, i] ^ 0x20
    assert follow_r1svd(A, one, S, 2, far["U_code"], far["V_code"], far["sigma"], 0.01)["U_code"][0, i] == \
        base["U_code"][0, i]
    # following one's own results changes nothing
    same = follow_r1svd(A, one, S, 2, base["U_code"], base["V_code"], base["sigma"], 0.01)
    assert same["followed"] == 0 and np.array_equal(same["A"], base["A"])
    # a forced sigma is what gets deflated
    sf = np.array([np.nan, base["sigma"][1] * 1.5])
    forced = ro.r1svd(A, S, 2, sigma_force=sf)
    assert forced["sigma"][0] == base["sigma"][0] and forced["sigma"][1] == sf[1]
    assert np.allclose(forced["A"], base["A"] - (sf[1] - base["sigma"][1]) * np.outer(base["U"][1], base["V"][1]))


def test_sigma_beyond_fp16_saturates_and_later_ranks_take_the_rest():
    # a rank-one matrix with singular value 150000 > 65504: three ranks of (about) 65504,
    # 65504 and the remainder rebuild it; an infinite sigma would have left NaN everywhere
    rng = np.random.default_rng(27)
    a = rng.standard_normal(24); a /= np.linalg.norm(a)
    b = rng.standard_normal(20); b /= np.linalg.norm(b)
    A = 150000.0 * np.outer(a, b)
    out = ro.r1svd(A, rng.standard_normal((4, 20)), 2)
    assert out["sigma"][0] == 65504.0 and np.all(np.isfinite(out["A"]))
    # the e4m3 factors are a little short of unit norm, so the first two ranks remove a little less
    assert out["sigma"][1] == 65504.0 and 0 < out["sigma"][2] < 65504.0
    assert np.linalg.norm(out["A"]) < 0.02 * 150000.0
    assert ro.fp16_round(65519.9) == 65504.0 and ro.fp16_round(1e9) == 65504.0
    assert ro.fp16_round(65503.0) == float(np.float16(65503.0))
