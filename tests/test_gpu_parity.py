"""GPU parity: every step of the hot path, called through the C ABI, against
the CPU oracle on the same seeded inputs.  Sizes are ones the oracle finishes
in seconds while still spanning several tiles and ragged tails.

Bars (from the benchmark spec):
  H                    relative error <= 1e-5 (Frobenius, and entry-wise scaled by sqrt(H_ii H_jj))
  U                    not stated; derived: float64 with a differently ordered
                       but backward-stable elimination, well-scaled H  ->  1e-9 of max|U|
  codes/scales/zeros   bit-exact, except decisions whose pre-rounding value lies
                       within 1e-5 of a rounding boundary (counted; see tests/parity.py)
  layer error          |rel_gpu - rel_oracle| <= 1e-4
"""
import math

import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq
import ptq_workloads as wl
from oracle import ptq_oracle as orc
from parity import compare_quantization, hessian_errors, to_device

pytestmark = pytest.mark.gpu


def _gpu_hessian(Xs, H=None):
    X = to_device(Xs)
    n = X.shape[1]
    if H is None:
        H = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    ptq.ptq_hessian_accumulate(H, X)
    return H


def _gpu_factor(H_np, damp, n=None):
    H = torch.from_numpy(np.ascontiguousarray(H_np)).cuda()
    n = H.shape[0]
    U = torch.full((n, n), float("nan"), dtype=torch.float64, device="cuda")
    dead = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    info = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ptq.ptq_damped_cholesky_inv(H, damp, U, dead, info)
    torch.cuda.synchronize()
    return U.cpu().numpy(), dead.cpu().numpy().astype(bool), info.cpu().numpy()


def _gpu_quantize(Ws, U_np, bits, group, block, dead=None, want_wq=True, static_groups=False):
    W = to_device(Ws)
    m, n = W.shape
    U = torch.from_numpy(np.ascontiguousarray(U_np)).cuda()
    codes = torch.full((m, n), 255, dtype=torch.uint8, device="cuda")
    scales = torch.full((m, n // group), float("nan"), dtype=torch.float32, device="cuda")
    zeros = torch.full((m, n // group), 255, dtype=torch.uint8, device="cuda")
    Wq = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda") if want_wq else None
    err2 = torch.full((m,), float("nan"), dtype=torch.float64, device="cuda")
    dm = None if dead is None else torch.from_numpy(dead.astype(np.uint8)).cuda()
    solve = ptq.ptq_quantize_layer_static_groups if static_groups else ptq.ptq_quantize_layer
    solve(W, U, dm, bits, group, block, codes, scales, zeros, Wq, err2)
    torch.cuda.synchronize()
    return dict(codes=codes.cpu().numpy(), scales=scales.cpu().numpy(), zeros=zeros.cpu().numpy(),
                Wq=None if Wq is None else Wq.cpu().numpy(), row_err2=err2.cpu().numpy())


def _correlated_x(rng, t, n, corr=0.8):
    A = rng.standard_normal((n, n))
    X = rng.standard_normal((t, n)) @ (np.eye(n) + corr * A / math.sqrt(n))
    return X * np.exp(rng.standard_normal(n))


# ------------------------------------------------------------------ Hessian
@pytest.mark.parametrize("dtype,t,n", [
    ("bf16", 1000, 384), ("bf16", 4096 + 17, 200), ("bf16", 300, 8), ("bf16", 9000, 136),
    ("bf16", 3000, 2304), ("bf16", 20000 + 5, 2056),      # wide layers: the 256 x 256-tile kernel
    ("bf16", 50, 2048), ("bf16", 1, 2048), ("bf16", 129, 2560),   # ... with fewer tokens than its LDS ring holds
    ("f32", 2048, 512), ("f32", 333, 70), ("f32", 5, 1),
    ("f32", 1500, 1024), ("f32", 9000 + 3, 1300),          # from 1024 channels on: 128 x 128 tiles, here ragged, two chunks
])
def test_hessian_matches_oracle(dtype, t, n):
    spec = wl.LayerSpec("h", 16, n, t, dtype=dtype, x_sigma=1.5, layer_id=900 + n)
    Xs = wl.gen_activations(spec)
    H = _gpu_hessian(Xs).cpu().numpy()
    Href = orc.hessian(wl.to_f64(Xs))
    fro, ent = hessian_errors(H, Href)
    print(f"H error: frobenius {fro:.2e}, scaled entry-wise {ent:.2e}")
    assert fro <= 1e-5 and ent <= 1e-5, (fro, ent)
    # f32 inputs are accumulated in float64 throughout
    if dtype == "f32":
        assert fro <= 1e-13


def test_hessian_accumulates_over_calls_and_is_reproducible():
    spec = wl.LayerSpec("h", 16, 256, 6000, dtype="bf16", layer_id=901)
    Xs = wl.gen_activations(spec)
    H1 = _gpu_hessian(Xs[:2500])
    H1 = _gpu_hessian(Xs[2500:], H1).cpu().numpy()
    Href = orc.hessian(wl.to_f64(Xs))
    fro, ent = hessian_errors(H1, Href)
    assert fro <= 1e-5 and ent <= 1e-5
    a = _gpu_hessian(Xs).cpu().numpy()
    b = _gpu_hessian(Xs).cpu().numpy()
    assert np.array_equal(np.triu(a), np.triu(b))
    # strided input (leading dimension larger than n)
    wide = np.zeros((6000, 320), dtype=np.uint16)
    wide[:, :256] = Xs
    Xw = to_device(wide)[:, :256]
    H = torch.zeros((256, 256), dtype=torch.float64, device="cuda")
    ptq.ptq_hessian_accumulate(H, Xw)
    assert np.array_equal(np.triu(H.cpu().numpy()), np.triu(a))
    # empty chunk is a no-op
    ptq.ptq_hessian_accumulate(H, Xw[:0])
    assert np.array_equal(np.triu(H.cpu().numpy()), np.triu(a))


def test_hessian_wide_layer_strided_and_chunked():
    # the 256 x 256-tile kernel on a view with a leading dimension larger than n, fed in two calls
    t, n, ld = 2100, 2048, 2048 + 72
    spec = wl.LayerSpec("h", 16, n, t, dtype="bf16", x_sigma=1.5, layer_id=902)
    Xs = wl.gen_activations(spec)
    wide = np.zeros((t, ld), dtype=np.uint16)
    wide[:, 8:8 + n] = Xs
    Xw = to_device(wide)[:, 8:8 + n]
    H = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    ptq.ptq_hessian_accumulate(H, Xw[:1037])
    ptq.ptq_hessian_accumulate(H, Xw[1037:])
    Href = orc.hessian(wl.to_f64(Xs))
    fro, ent = hessian_errors(H.cpu().numpy(), Href)
    assert fro <= 1e-5 and ent <= 1e-5, (fro, ent)
    a = _gpu_hessian(Xs).cpu().numpy()
    b = _gpu_hessian(Xs).cpu().numpy()
    assert np.array_equal(np.triu(a), np.triu(b))


# ------------------------------------------------------------------ factor
@pytest.mark.parametrize("n", [1, 17, 128, 200, 257, 512, 1000])
def test_factor_matches_oracle(n):
    rng = np.random.default_rng(n)
    X = _correlated_x(rng, 2 * n + 3, n)
    H = orc.hessian(X)
    Hd, dead_ref = orc.damp(H, 0.01)
    Uref = orc.inverse_cholesky_upper(Hd)
    # the library reads only the upper triangle: poison the lower one
    Hin = np.triu(H) + np.tril(np.full((n, n), 1e30), -1)
    U, dead, info = _gpu_factor(Hin, 0.01)
    assert info.tolist() == [0, 0] and not dead.any()
    assert np.all(np.tril(U, -1) == 0) and np.all(np.diag(U) > 0)
    assert np.max(np.abs(U - Uref)) <= 1e-9 * np.max(np.abs(Uref))
    assert np.allclose(U.T @ U @ Hd, np.eye(n), rtol=0, atol=1e-7)


def test_factor_dead_channel_and_not_spd():
    rng = np.random.default_rng(3)
    n = 96
    X = _correlated_x(rng, 300, n)
    X[:, 40] = 0.0
    H = orc.hessian(X)
    Hd, dead_ref = orc.damp(H, 0.05)
    U, dead, info = _gpu_factor(np.triu(H), 0.05)
    assert info.tolist() == [0, 0] and np.array_equal(dead, dead_ref) and dead[40]
    Uref = orc.inverse_cholesky_upper(Hd)
    assert np.max(np.abs(U - Uref)) <= 1e-9 * np.max(np.abs(Uref))
    # an indefinite matrix: the elimination runs from the last index down and
    # reports the first non-positive pivot in H's own indexing
    Hbad = np.diag(np.linspace(1.0, 2.0, n))
    Hbad[10, 10] = -1.0
    _, _, info = _gpu_factor(Hbad, 0.0)
    assert info.tolist() == [5, 10]


# ------------------------------------------------------------------ solve
CASES = [
    # name, dtype, m, n, t, bits, group, block
    ("c1_like", "f32", 512, 512, 2048, 4, 128, 128),
    ("ragged_rows_3bit", "bf16", 70, 384, 1200, 3, 64, 128),
    ("two_bit_b256", "bf16", 48, 512, 1500, 2, 64, 256),
    ("eight_bit", "bf16", 33, 256, 800, 8, 32, 64),
    ("block_tail", "f32", 40, 384, 1000, 4, 128, 256),
    ("group_wider_than_block", "bf16", 24, 512, 1300, 3, 128, 64),
    ("tiny", "f32", 1, 16, 40, 4, 16, 16),
    # tall layers: two and three 16-row tiles per workgroup, with a ragged last workgroup
    ("tall_two_row_tiles", "bf16", 4700, 256, 700, 3, 128, 128),
    ("tall_three_row_tiles", "bf16", 9300, 192, 600, 4, 64, 64),
    ("tall_three_row_tiles_b256", "f32", 9237, 320, 900, 2, 64, 256),
]


def _layer(name, dtype, m, n, t, correlated, seed):
    spec = wl.LayerSpec(name, m, n, t, dtype=dtype, outlier_frac=0.01, outlier_mul=10.0, layer_id=seed)
    Ws = wl.gen_weight(spec)
    if correlated:
        rng = np.random.default_rng(seed)
        X = _correlated_x(rng, t, n)
    else:
        X = wl.to_f64(wl.gen_activations(spec))
    return Ws, X


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("correlated", [False, True], ids=["iid", "correlated"])
def test_quantize_matches_oracle(case, correlated):
    name, dtype, m, n, t, bits, group, block = case
    Ws, X = _layer(name, dtype, m, n, t, correlated, 700 + len(name))
    H = orc.hessian(X)
    Hd, _ = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    g = _gpu_quantize(Ws, U, bits, group, block)
    W64 = wl.to_f64(Ws)
    rep = compare_quantization(W64, U, bits, group, None, g["codes"], g["scales"], g["zeros"])
    print(f"{name}: exact rows {rep['exact_rows']}/{m}, flagged c/z/s = {rep['flagged_codes']}/"
          f"{rep['flagged_zeros']}/{rep['flagged_scales']}, unflagged {rep['unflagged']}")
    assert rep["unflagged"] == 0, rep["details"][:5]
    # with the oracle's own U only summation order differs: near-ties must be rare
    assert rep["flagged_codes"] + rep["flagged_zeros"] + rep["flagged_scales"] <= max(2, m * n // 100000)
    assert rep["max_scale_margin_ulp"] <= 1e-3
    if rep["exact_rows"] == m:
        o = rep["oracle"]
        assert np.allclose(g["Wq"], o["Wq"], rtol=0, atol=0)
        assert np.allclose(g["row_err2"], o["row_err2"], rtol=1e-9, atol=1e-30)
    assert np.array_equal(g["Wq"], orc.dequantize(g["codes"], g["scales"], g["zeros"], group))


@pytest.mark.parametrize("case", [CASES[1], CASES[2], CASES[4], CASES[5]], ids=lambda c: c[0])
def test_quantize_with_static_groups_matches_oracle(case):
    """Every group's grid from the weights as given: same protocol as the ordinary solve."""
    name, dtype, m, n, t, bits, group, block = case
    Ws, X = _layer(name, dtype, m, n, t, True, 800 + len(name))
    U = orc.inverse_cholesky_upper(orc.damp(orc.hessian(X), 0.01)[0])
    dead = np.zeros(n, dtype=bool)
    dead[[3, n // 2]] = True          # dead columns count as zeros in the grids too
    g = _gpu_quantize(Ws, U, bits, group, block, dead=dead, static_groups=True)
    W64 = wl.to_f64(Ws)
    rep = compare_quantization(W64, U, bits, group, dead, g["codes"], g["scales"], g["zeros"], static_groups=True)
    assert rep["unflagged"] == 0, rep["details"][:5]
    assert rep["flagged_codes"] + rep["flagged_zeros"] + rep["flagged_scales"] <= 2
    # the grids are those of round-to-nearest on the given weights, whatever the Hessian did to the codes
    Wz = W64.copy()
    Wz[:, dead] = 0.0
    rtn = orc.round_to_nearest(Wz, bits, group)
    assert np.array_equal(g["scales"], rtn["scales"]) and np.array_equal(g["zeros"], rtn["zeros"])
    assert np.array_equal(g["Wq"], orc.dequantize(g["codes"], g["scales"], g["zeros"], group))
    dyn = _gpu_quantize(Ws, U, bits, group, block, dead=dead)
    assert not np.array_equal(dyn["scales"], g["scales"])


def test_quantize_block_size_changes_nothing():
    Ws, X = _layer("blk", "bf16", 64, 512, 1500, True, 777)
    U = orc.inverse_cholesky_upper(orc.damp(orc.hessian(X), 0.01)[0])
    outs = [_gpu_quantize(Ws, U, 4, 64, b) for b in (64, 128, 256)]
    W64 = wl.to_f64(Ws)
    for o in outs:
        rep = compare_quantization(W64, U, 4, 64, None, o["codes"], o["scales"], o["zeros"])
        assert rep["unflagged"] == 0
    # the three block sizes agree wherever no near-tie was flagged (normally everywhere)
    same = [np.array_equal(outs[0]["codes"], o["codes"]) for o in outs[1:]]
    print("block-size invariance exact:", same)


def test_quantize_on_grid_recovery_and_diagonal_hessian():
    rng = np.random.default_rng(8)
    m, n, group, bits = 40, 256, 64, 4
    maxq = 15
    codes = rng.integers(0, maxq + 1, size=(m, n))
    ng = n // group
    scales = 2.0 ** rng.integers(-8, -2, size=(m, ng))
    zeros = rng.integers(1, maxq, size=(m, ng))
    for r in range(m):
        for k in range(ng):
            a, b = rng.choice(group, 2, replace=False)
            codes[r, k * group + a] = 0
            codes[r, k * group + b] = maxq
    W = np.repeat(scales, group, axis=1) * (codes - np.repeat(zeros, group, axis=1))
    X = _correlated_x(rng, 600, n)
    U = orc.inverse_cholesky_upper(orc.damp(orc.hessian(X), 0.01)[0])
    g = _gpu_quantize(W, U, bits, group, 128)
    assert np.array_equal(g["codes"], codes) and np.array_equal(g["zeros"], zeros)
    assert np.array_equal(g["scales"].astype(np.float64), scales)
    assert np.array_equal(g["Wq"], W) and np.all(g["row_err2"] == 0)
    # diagonal H: no compensation, the result is plain round-to-nearest
    Wr = rng.standard_normal((m, n)) * 0.02
    Ud = np.diag(1 / np.sqrt(rng.uniform(0.5, 50.0, n)))
    g = _gpu_quantize(Wr, Ud, 3, group, 128)
    rtn = orc.round_to_nearest(Wr, 3, group)
    assert np.array_equal(g["codes"], rtn["codes"]) and np.array_equal(g["scales"], rtn["scales"])
    assert np.array_equal(g["zeros"], rtn["zeros"])


def test_quantize_dead_channel_and_exact_ties():
    rng = np.random.default_rng(9)
    m, n, group, bits = 20, 128, 32, 4
    X = _correlated_x(rng, 400, n)
    X[:, 17] = 0.0
    H = orc.hessian(X)
    Hd, dead = orc.damp(H, 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    W = rng.standard_normal((m, n)) * 0.02
    W[:, 17] = 3.0
    g = _gpu_quantize(W, U, bits, group, 64, dead=dead)
    rep = compare_quantization(W, U, bits, group, dead, g["codes"], g["scales"], g["zeros"])
    assert rep["unflagged"] == 0 and np.all(g["Wq"][:, 17] == 0)
    # exact half-way values round to even exactly as in the oracle (identity U)
    Wt = np.zeros((4, 32))
    Wt[:, 0] = -1.0
    Wt[:, 1] = 14.0                       # range 15 -> scale 1, zero 1
    Wt[:, 2:] = np.arange(30) * 0.5 - 1.0  # many exact .5 values
    g = _gpu_quantize(Wt, np.eye(32), 4, 32, 32)
    o = orc.quantize_layer(Wt, np.eye(32), 4, 32)
    assert np.array_equal(g["codes"], o["codes"]) and np.array_equal(g["zeros"], o["zeros"])


# ------------------------------------------------------------------ layer error
@pytest.mark.parametrize("dtype,m,n", [("bf16", 300, 384), ("f32", 70, 200), ("f64", 129, 130), ("f32", 1, 1),
                                       ("bf16", 513, 1000), ("bf16", 128, 128)])
def test_layer_error_matches_oracle(dtype, m, n):
    rng = np.random.default_rng(m)
    X = _correlated_x(rng, 2 * n, n)
    H = orc.hessian(X)
    W64 = rng.standard_normal((m, n)) * 0.02
    Ws = wl.store(W64, dtype)
    W64 = wl.to_f64(Ws)
    Wq = W64 + 0.003 * rng.standard_normal((m, n))
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    Hin = np.triu(H) + np.tril(np.full((n, n), 1e30), -1)
    ptq.ptq_layer_error(to_device(Ws), torch.from_numpy(Wq).cuda(), torch.from_numpy(Hin).cuda(), out)
    rel, num, den = out.cpu().numpy()
    r0, n0, d0 = orc.layer_error(W64, Wq, H)
    # float64 weights: float64 throughout.  float32 / bfloat16 weights, fewer than 65536 entries: D, W and
    # H rounded to float32, products (from three bfloat16 pieces, complete to 2^-24) and sums over k in
    # float32 on the matrix cores -- four roundings of 2^-24 per term at worst (that worst case is the
    # 1 x 1 layer), far less once m n terms average them out.  From 65536 entries on, two pieces: terms
    # complete to 2^-16, unbiased, and the traces average m n of them -- the required agreement is 1e-4
    # on the relative error; held here to 3e-7 on it and to 4e-6 on the two traces.
    tol = 1e-10 if dtype == "f64" else 3e-7
    tol_trace = tol if (dtype == "f64" or m * n < 65536) else 4e-6
    assert abs(rel - r0) <= 1e-4 and abs(rel - r0) <= tol
    assert abs(num - n0) <= tol_trace * n0 and abs(den - d0) <= tol_trace * d0


# ------------------------------------------------------------------ end to end
def test_end_to_end_small_fp32_layer():
    """The first benchmark configuration (512 x 512 fp32, 2048 tokens), every
    step on the GPU, against the oracle chain on the same bits."""
    cfg = wl.CONFIGS["C1"]
    spec = cfg.layers[0]
    Ws, Xs = wl.gen_weight(spec), wl.gen_activations(spec)
    W64, X64 = wl.to_f64(Ws), wl.to_f64(Xs)
    Href = orc.hessian(X64)
    Hd, dead_ref = orc.damp(Href, cfg.damps[0])
    Uref = orc.inverse_cholesky_upper(Hd)

    n = spec.n
    H = _gpu_hessian(Xs)
    U = torch.empty((n, n), dtype=torch.float64, device="cuda")
    dead = torch.empty((n,), dtype=torch.uint8, device="cuda")
    info = torch.empty((2,), dtype=torch.int32, device="cuda")
    ptq.ptq_damped_cholesky_inv(H, cfg.damps[0], U, dead, info)
    W = to_device(Ws)
    m = spec.m
    codes = torch.empty((m, n), dtype=torch.uint8, device="cuda")
    scales = torch.empty((m, n // cfg.group), dtype=torch.float32, device="cuda")
    zeros = torch.empty((m, n // cfg.group), dtype=torch.uint8, device="cuda")
    Wq = torch.empty((m, n), dtype=torch.float64, device="cuda")
    ptq.ptq_quantize_layer(W, U, dead, cfg.bits, cfg.group, cfg.block, codes, scales, zeros, Wq, None)
    out = torch.zeros(3, dtype=torch.float64, device="cuda")
    ptq.ptq_layer_error(W, Wq, H, out)
    torch.cuda.synchronize()

    fro, ent = hessian_errors(H.cpu().numpy(), Href)
    assert fro <= 1e-5 and ent <= 1e-5
    assert info.cpu().tolist() == [0, 0]
    assert np.max(np.abs(U.cpu().numpy() - Uref)) <= 1e-9 * np.max(np.abs(Uref))
    rep = compare_quantization(W64, Uref, cfg.bits, cfg.group, None, codes.cpu().numpy(),
                               scales.cpu().numpy(), zeros.cpu().numpy())
    print(f"C1 end to end: exact rows {rep['exact_rows']}/{m}, flagged c/z/s = {rep['flagged_codes']}/"
          f"{rep['flagged_zeros']}/{rep['flagged_scales']}, unflagged {rep['unflagged']}")
    assert rep["unflagged"] == 0
    rel_ref = orc.layer_error(W64, rep["oracle"]["Wq"], Href)[0]
    rel_rtn = orc.layer_error(W64, orc.round_to_nearest(W64, cfg.bits, cfg.group)["Wq"], Href)[0]
    rel = float(out[0])
    assert abs(rel - rel_ref) <= 1e-4
    assert rel <= rel_rtn


def test_step_can_be_captured_in_a_graph_and_replayed():
    """The four calls of the path enqueue kernels only (no allocation, no memset, no synchronization), so a
    whole step can be captured in a HIP graph.  Replays with new activations in the same buffer must match
    the eager calls exactly."""
    m, n, t, bits, group, block = 64, 512, 1536, 4, 128, 128
    spec = wl.LayerSpec("graph", m, n, t, dtype="bf16", x_sigma=1.0, layer_id=1400)
    Wd = to_device(wl.gen_weight(spec))
    Xs = [to_device(wl.gen_activations(wl.LayerSpec("graph", m, n, t, dtype="bf16", x_sigma=1.0, layer_id=1400 + k)))
          for k in range(3)]
    d = "cuda"
    X = torch.empty_like(Xs[0])
    H = torch.zeros((n, n), dtype=torch.float64, device=d)
    U = torch.empty((n, n), dtype=torch.float64, device=d)
    dead = torch.empty(n, dtype=torch.uint8, device=d)
    info = torch.empty(2, dtype=torch.int32, device=d)
    codes = torch.empty((m, n), dtype=torch.uint8, device=d)
    scales = torch.empty((m, n // group), dtype=torch.float32, device=d)
    zeros = torch.empty((m, n // group), dtype=torch.uint8, device=d)
    Wq = torch.empty((m, n), dtype=torch.float64, device=d)
    out = torch.zeros(3, dtype=torch.float64, device=d)
    ws = torch.empty(max(ptq.ptq_workspace_bytes(op, m, n, t, block) for op in range(4)), dtype=torch.uint8, device=d)

    def step():
        H.zero_()
        ptq.ptq_hessian_accumulate(H, X, ws)
        ptq.ptq_damped_cholesky_inv(H, 0.01, U, dead, info, ws)
        ptq.ptq_quantize_layer(Wd, U, dead, bits, group, block, codes, scales, zeros, Wq, None, ws)
        ptq.ptq_layer_error(Wd, Wq, H, out, ws)

    eager = []
    for Xk in Xs:                       # eager results first (this also warms every kernel up)
        X.copy_(Xk)
        step()
        torch.cuda.synchronize()
        eager.append((codes.clone(), scales.clone(), zeros.clone(), out.clone()))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        X.copy_(Xs[0])
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for k in (1, 2, 0, 1):              # replays, with eager work and synchronization in between
        X.copy_(Xs[k])
        codes.zero_()
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert info.cpu().tolist() == [0, 0]
        assert torch.equal(codes, eager[k][0]) and torch.equal(scales, eager[k][1])
        assert torch.equal(zeros, eager[k][2]) and torch.equal(out, eager[k][3])
