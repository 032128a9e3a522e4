"""GPU parity of the stored form of a layer (bit packing, dequantization) and of the layer applied
to a few tokens in the rotated-input form of Eq. 7, against oracle/artifact_oracle.py."""
import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq
from oracle import artifact_oracle as ao
from oracle import lopro_oracle as lo
from oracle import r1svd_oracle as ro

pytestmark = pytest.mark.gpu

# float32 sums: a lane adds the 32 products of a chunk in sequence, the chunk sums of a run, then the
# runs and the low-rank terms in sequence, plus one rounding each for X~, the grid and the coefficients
def _gamma(n):
    return (32 + 8 + n // 256 + 80) * 2.0 ** -24


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
@pytest.mark.parametrize("m,n", [(37, 160), (5, 4096)])
def test_pack_matches_oracle_and_unpacks(bits, m, n):
    rng = np.random.default_rng(bits * 100 + m)
    codes = rng.integers(0, 2 ** bits, size=(m, n), dtype=np.uint8)
    group = 32
    scales = rng.uniform(0.001, 0.2, size=(m, n // group)).astype(np.float32)
    zeros = rng.integers(0, 2 ** bits, size=(m, n // group), dtype=np.uint8)
    packed = torch.full((n // 32, m, bits), -1, dtype=torch.int32, device="cuda")
    st = torch.full((n // group, m), float("nan"), dtype=torch.float32, device="cuda")
    zt = torch.full((n // group, m), 0xEE, dtype=torch.uint8, device="cuda")
    ptq.ptq_pack_codes(_dev(codes), bits, packed, _dev(scales), _dev(zeros), group, st, zt)
    got = packed.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, ao.pack_codes(codes, bits))
    assert np.array_equal(st.cpu().numpy(), scales.T) and np.array_equal(zt.cpu().numpy(), zeros.T)
    only = torch.full_like(packed, -1)
    ptq.ptq_pack_codes(_dev(codes), bits, only)           # codes alone
    assert torch.equal(only, packed)
    Wq = torch.full((m, n), float("nan"), dtype=torch.float64, device="cuda")
    ptq.ptq_unpack_dequantize(packed, n, bits, st, zt, group, Wq)
    assert np.array_equal(Wq.cpu().numpy(), ao.dequantize(codes, scales, zeros, group))


def test_unpack_reproduces_what_the_solve_wrote():
    import ptq_workloads as wl
    from oracle import ptq_oracle as orc
    from parity import to_device
    m, n, bits, group = 40, 512, 3, 64
    spec = wl.LayerSpec("pk", m, n, 1024, dtype="f32", x_sigma=1.0, layer_id=1201)
    Ws, Xs = wl.gen_weight(spec), wl.gen_activations(spec)
    H = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    ptq.ptq_hessian_accumulate(H, to_device(Xs))
    U, dead, info = (torch.empty((n, n), dtype=torch.float64, device="cuda"),
                     torch.empty(n, dtype=torch.uint8, device="cuda"), torch.empty(2, dtype=torch.int32, device="cuda"))
    ptq.ptq_damped_cholesky_inv(H, 0.01, U, dead, info)
    codes = torch.empty((m, n), dtype=torch.uint8, device="cuda")
    scales = torch.empty((m, n // group), dtype=torch.float32, device="cuda")
    zeros = torch.empty((m, n // group), dtype=torch.uint8, device="cuda")
    Wq = torch.empty((m, n), dtype=torch.float64, device="cuda")
    ptq.ptq_quantize_layer(to_device(Ws), U, dead, bits, group, 128, codes, scales, zeros, Wq, None)
    packed = torch.empty((n // 32, m, bits), dtype=torch.int32, device="cuda")
    st = torch.empty((n // group, m), dtype=torch.float32, device="cuda")
    zt = torch.empty((n // group, m), dtype=torch.uint8, device="cuda")
    ptq.ptq_pack_codes(codes, bits, packed, scales, zeros, group, st, zt)
    back = torch.empty_like(Wq)
    ptq.ptq_unpack_dequantize(packed, n, bits, st, zt, group, back)
    assert torch.equal(back, Wq)
    assert packed.numel() * 32 == m * n * bits


def _random_layer(rng, m, n, r, bits, group):
    codes = rng.integers(0, 2 ** bits, size=(m, n), dtype=np.uint8)
    scales = rng.uniform(0.002, 0.05, size=(m, n // group)).astype(np.float32)
    zeros = rng.integers(0, 2 ** bits, size=(m, n // group), dtype=np.uint8)
    perm = rng.permutation(n).astype(np.int32)
    u = rng.standard_normal((r, m)); u /= np.linalg.norm(u, axis=1, keepdims=True)
    v = rng.standard_normal((r, n)); v /= np.linalg.norm(v, axis=1, keepdims=True)
    Uc, Vc = ro.e4m3_encode(ro.e4m3_round(u)[0]), ro.e4m3_encode(ro.e4m3_round(v)[0])
    sigma = np.sort(rng.uniform(1.0, 40.0, r))[::-1].astype(np.float16)
    s = np.exp(rng.normal(0, 0.7, n))
    return codes, scales, zeros, perm, Uc, Vc, sigma, s


def _forward(X_t, codes, scales, zeros, perm, Uc, Vc, sigma, s, bits, group, bI, bH):
    m, n = codes.shape
    tokens = X_t.shape[0]
    packed = torch.empty((n // 32, m, bits), dtype=torch.int32, device="cuda")
    st = torch.empty((n // group, m), dtype=torch.float32, device="cuda")
    zt = torch.empty((n // group, m), dtype=torch.uint8, device="cuda")
    ptq.ptq_pack_codes(_dev(codes), bits, packed, _dev(scales), _dev(zeros), group, st, zt)
    O = torch.full((tokens, m), float("nan"), dtype=torch.float32, device="cuda")
    r = Uc.shape[0]
    ptq.ptq_lopro_linear_forward(X_t, packed, bits, st, zt, group, _dev(perm), bI, bH,
                                 _dev(Uc) if r else None, _dev(Vc) if r else None,
                                 torch.from_numpy(sigma.copy()).cuda() if r else None, _dev(s) if r else None, O)
    torch.cuda.synchronize()
    return O.cpu().numpy().astype(np.float64), packed.cpu().numpy().view(np.uint32)


def _check_forward(X64, got, packed, codes, scales, zeros, perm, Uc, Vc, sigma, s, bits, group, bI, bH):
    n = X64.shape[1]
    p64 = perm.astype(np.int64)
    sig = sigma.astype(np.float64)
    ref = ao.linear_forward(X64, packed, bits, scales, zeros, group, p64, bI, bH, Uc, Vc, sig, s)
    Xt = lo.rotate_weight(X64, p64, bI, bH)
    # the kernel sums scale * code * x and scale * zero * x separately (the second does not depend on the row)
    sc = np.repeat(scales.astype(np.float64), group, axis=1)
    zz = np.repeat(zeros.astype(np.float64), group, axis=1)
    mag = np.abs(Xt) @ (sc * (codes.astype(np.float64) + zz)).T
    if Uc.shape[0]:
        mag += (np.abs(X64 / s) @ np.abs(ro.e4m3_decode(Vc)).T * sig) @ np.abs(ro.e4m3_decode(Uc))
    err = np.abs(got - ref)
    tol = _gamma(n) * mag + 1e-30
    assert np.all(err <= tol), float(np.max(err / tol))
    return ref


@pytest.mark.parametrize("bits,tokens,dtype,r", [(2, 1, torch.float32, 4), (3, 3, torch.bfloat16, 5),
                                                 (4, 7, torch.float32, 16), (8, 2, torch.float64, 0),
                                                 (3, 4, torch.float32, 70), (4, 29, torch.bfloat16, 16),
                                                 (2, 16, torch.float32, 3)])
def test_forward_matches_oracle(bits, tokens, dtype, r):
    rng = np.random.default_rng(bits * 10 + tokens)
    m, n, group, bI, bH = 77, 1024, 64, 256, 128
    layer = _random_layer(rng, m, n, r, bits, group)
    X_t = _dev(rng.standard_normal((tokens, n))).to(dtype)
    X64 = X_t.to(torch.float64).cpu().numpy()
    got, packed = _forward(X_t, *layer, bits, group, bI, bH)
    _check_forward(X64, got, packed, *layer, bits, group, bI, bH)


@pytest.mark.parametrize("bits,tokens,m,group", [(4, 19, 256, 128), (3, 32, 132, 32), (2, 45, 64, 512)])
def test_forward_many_tokens_on_the_matrix_cores(bits, tokens, m, group):
    """Eight or more tokens go through the float32 MFMA kernel, up to 32 per pass; groups of one chunk,
    of four, and longer than a workgroup's run of columns; m a multiple of 4 (wide loads in the finish)."""
    rng = np.random.default_rng(1000 + tokens)
    n, bI, bH, r = 1024, 256, 128, 6
    layer = _random_layer(rng, m, n, r, bits, group)
    X_t = _dev(rng.standard_normal((tokens, n)).astype(np.float32))
    X64 = X_t.to(torch.float64).cpu().numpy()
    got, packed = _forward(X_t, *layer, bits, group, bI, bH)
    _check_forward(X64, got, packed, *layer, bits, group, bI, bH)


def test_forward_without_rotation_or_low_rank_is_a_plain_dequantized_product():
    rng = np.random.default_rng(7)
    m, n, bits, group = 33, 512, 4, 128
    codes, scales, zeros, _, Uc, Vc, sigma, s = _random_layer(rng, m, n, 0, bits, group)
    perm = np.arange(n, dtype=np.int32)
    X_t = _dev(rng.standard_normal((2, n)).astype(np.float32))
    got, _ = _forward(X_t, codes, scales, zeros, perm, Uc, Vc, sigma, s, bits, group, n, 256)
    ref = X_t.to(torch.float64).cpu().numpy() @ ao.dequantize(codes, scales, zeros, group).T
    assert np.allclose(got, ref, rtol=0, atol=_gamma(n) * np.max(np.abs(ref)) * 100)


@pytest.mark.parametrize("tokens", [4, 45])   # 45 = a matrix-core pass of 32, one of 13: both kernels at full size
def test_forward_full_size_attention_projection(tokens):
    rng = np.random.default_rng(99)
    m = n = 4096
    bits, group, bI, bH, r = 3, 128, 256, 256, 16
    layer = _random_layer(rng, m, n, r, bits, group)
    X_t = _dev(rng.standard_normal((tokens, n)).astype(np.float32)).to(torch.bfloat16)
    got, packed = _forward(X_t, *layer, bits, group, bI, bH)
    _check_forward(X_t.to(torch.float64).cpu().numpy(), got, packed, *layer, bits, group, bI, bH)
