"""GPU parity of the vector-quantized solve (ptq_quantize_layer_vq) against oracle/vq_oracle.py:
indices bit-exact except counted near-ties of the assignment (tests/parity.py, compare_vq), the
assigned values, the errors' identity, small ragged shapes and the full 4096 x 4096 layer in the
paper's two settings (4-D vectors, 256 entries; 2-D vectors, 64 entries)."""
import time

import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq
import ptq_workloads as wl
from oracle import ptq_oracle as orc
from oracle import vq_oracle as vqo
from parity import compare_vq, to_device

pytestmark = pytest.mark.gpu


def _correlated_x(rng, t, n):
    A = np.eye(n) + 0.8 * rng.standard_normal((n, n)) / np.sqrt(n)
    return (rng.standard_normal((t, n)) @ A) * np.exp(rng.normal(0.0, 1.0, n))[None, :]


def _gpu_vq(Ws, U, C, block, dead=None):
    W = to_device(Ws)
    m, n = W.shape
    K, d = C.shape
    idx = torch.full((m, n // d), 0xEE, dtype=torch.uint8, device="cuda")
    Wq = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    e2 = torch.full((m,), float("nan"), dtype=torch.float64, device="cuda")
    dm = None if dead is None else torch.from_numpy(dead.astype(np.uint8)).cuda()
    ptq.ptq_quantize_layer_vq(W, torch.from_numpy(U).cuda(), dm, torch.from_numpy(C).cuda(), block, idx, Wq, e2)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), Wq.cpu().numpy(), e2.cpu().numpy()


CASES = [
    # name, dtype, m, n, t, entries, dim, block
    ("four_dim_256", "bf16", 70, 384, 1200, 256, 4, 128),
    ("two_dim_64", "bf16", 48, 512, 1500, 64, 2, 256),
    ("one_dim_16", "f32", 33, 256, 800, 16, 1, 64),
    ("odd_entries", "f32", 40, 384, 1000, 37, 4, 256),    # entries not a multiple of 32, a block tail
    ("few_entries", "bf16", 17, 128, 500, 5, 2, 128),
    ("tiny", "f32", 1, 16, 40, 3, 4, 16),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_vq_matches_oracle(case):
    name, dtype, m, n, t, K, d, block = case
    spec = wl.LayerSpec(name, m, n, t, dtype=dtype, outlier_frac=0.01, outlier_mul=10.0, layer_id=1400 + len(name))
    Ws = wl.gen_weight(spec)
    W64 = wl.to_f64(Ws)
    X = _correlated_x(np.random.default_rng(1400 + len(name)), t, n)
    Hd, _ = orc.damp(orc.hessian(X), 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    C = wl.gen_codebook(W64, K, d, spec)
    idx, Wq, e2 = _gpu_vq(Ws, U, C, block)
    rep = compare_vq(W64, U, C, None, idx)
    print(f"{name}: exact rows {rep['exact_rows']}/{m}, flagged {rep['flagged']}, unflagged {rep['unflagged']}")
    assert rep["unflagged"] == 0, rep["details"][:5]
    assert rep["flagged"] <= 1
    assert idx.max() < K
    assert np.array_equal(Wq, C.astype(np.float64)[idx].reshape(m, n))
    if rep["exact_rows"] == m:
        assert np.allclose(e2, rep["oracle"]["row_err2"], rtol=1e-9, atol=1e-300)
    D = W64 - Wq
    assert np.allclose(np.einsum("ij,ij->i", D @ Hd, D), e2, rtol=1e-8)


def test_vq_special_cases_on_the_gpu():
    rng = np.random.default_rng(15)
    m, n, d, K = 24, 128, 4, 32
    # weights made of codebook entries are recovered exactly, whatever the Hessian
    C = rng.standard_normal((K, d)).astype(np.float32)
    want = rng.integers(0, K, size=(m, n // d))
    W = C[want].reshape(m, n).astype(np.float32)
    U = orc.inverse_cholesky_upper(orc.damp(orc.hessian(_correlated_x(rng, 400, n)), 0.01)[0])
    idx, Wq, e2 = _gpu_vq(W, U, C, 64)
    assert np.array_equal(idx, want) and np.array_equal(Wq, W.astype(np.float64)) and not e2.any()
    # identity Hessian: the plain Euclidean nearest entry of the given weights
    W2 = rng.standard_normal((m, n)).astype(np.float32)
    idx, _, _ = _gpu_vq(W2, np.eye(n), C, 128)
    assert np.array_equal(idx, vqo.nearest_entries(W2.astype(np.float64), C))
    # a dead channel counts as zero; duplicated entries resolve to the lower index
    dead = np.zeros(n, dtype=bool); dead[[5, 64]] = True
    C2 = np.vstack([C[:8], C[:8]]).astype(np.float32)
    idx, _, _ = _gpu_vq(W2, U, C2, 128, dead=dead)
    rep = compare_vq(W2.astype(np.float64), U, C2, dead, idx)
    assert rep["unflagged"] == 0 and rep["flagged"] == 0 and idx.max() < 8


@pytest.mark.parametrize("K,d", [(256, 4), (64, 2)])
def test_vq_full_size_attention_projection(K, d, capsys):
    """4096 x 4096 at the launch shape bench.py uses, the oracle's factor of an 8192-token Hessian, 64 sampled rows."""
    cfg = wl.CONFIGS["C2"]
    spec = wl.scaled(cfg.layers[0], t=8192)
    Ws, Xs = wl.gen_weight(spec), wl.gen_activations(spec)
    W64 = wl.to_f64(Ws)
    Hd, _ = orc.damp(orc.hessian(wl.to_f64(Xs)), 0.01)
    U = orc.inverse_cholesky_upper(Hd)
    C = wl.gen_codebook(W64, K, d, spec)
    t0 = time.time()
    idx, Wq, e2 = _gpu_vq(Ws, U, C, cfg.block)
    rows = np.sort(np.random.default_rng(K).choice(spec.m, 64, replace=False))
    rows[0], rows[-1] = 0, spec.m - 1
    rep = compare_vq(W64[rows], U, C, None, idx[rows])
    with capsys.disabled():
        print(f"  [vq {K} x {d}: sampled rows exact {rep['exact_rows']}/64, flagged {rep['flagged']}, unflagged "
              f"{rep['unflagged']}; {time.time() - t0:.1f} s]", flush=True)
    assert rep["unflagged"] == 0, rep["details"][:5]
    assert rep["flagged"] <= 2
    assert np.array_equal(Wq, C.astype(np.float64)[idx].reshape(spec.m, spec.n))
    D = W64 - Wq
    assert np.allclose(np.einsum("ij,ij->i", D @ Hd, D), e2, rtol=1e-7)
