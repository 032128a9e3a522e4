"""The entry point that allocates nothing (ptq_lopro_linear_forward_static): same results as
ptq_lopro_linear_forward with a caller workspace, on two calls in a row that share the library's
per-GPU scratch array, the second with a smaller problem; sizes beyond the array are refused."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq

pytestmark = pytest.mark.gpu


def _layer(seed, m, n, r, bits, group, tokens, dtype):
    g = torch.Generator(device="cuda").manual_seed(seed)
    dev = "cuda"
    codes = torch.randint(0, 2 ** bits, (m, n), generator=g, device=dev, dtype=torch.uint8)
    scales = torch.rand((m, n // group), generator=g, device=dev) * 0.05 + 0.002
    zeros = torch.randint(0, 2 ** bits, (m, n // group), generator=g, device=dev, dtype=torch.uint8)
    packed = torch.empty((n // 32, m, bits), dtype=torch.int32, device=dev)
    st = torch.empty((n // group, m), dtype=torch.float32, device=dev)
    zt = torch.empty((n // group, m), dtype=torch.uint8, device=dev)
    ptq.ptq_pack_codes(codes, bits, packed, scales, zeros, group, st, zt)
    perm = torch.randperm(n, generator=g, device=dev).to(torch.int32)
    U = torch.randint(0x20, 0x38, (r, m), generator=g, device=dev, dtype=torch.uint8) if r else None
    V = torch.randint(0x20, 0x38, (r, n), generator=g, device=dev, dtype=torch.uint8) if r else None
    sg = (torch.rand(r, generator=g, device=dev) + 0.5).to(torch.float16) if r else None
    s = torch.exp(torch.randn(n, generator=g, device=dev, dtype=torch.float64)) if r else None
    X = torch.randn((tokens, n), generator=g, device=dev).to(dtype)
    return dict(X=X, packed=packed, bits=bits, st=st, zt=zt, group=group, perm=perm, U=U, V=V, sg=sg, s=s, m=m)


def _both(L, b_I, b_H):
    tokens = L["X"].shape[0]
    want = torch.full((tokens, L["m"]), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full_like(want, float("nan"))
    a = (L["X"], L["packed"], L["bits"], L["st"], L["zt"], L["group"], L["perm"], b_I, b_H, L["U"], L["V"], L["sg"],
         L["s"])
    ptq.ptq_lopro_linear_forward(*a, want)
    ptq.ptq_lopro_linear_forward_static(*a, got)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_forward_matches_the_workspace_form_twice_in_a_row():
    # first call: a 7B-sized attention projection, 16 tokens (matrix-core pass), rank-16 low-rank part;
    # second call, smaller in every size, on the same scratch array: few-token pass, no low-rank part
    big = _layer(1, 4096, 4096, 16, 4, 128, 16, torch.bfloat16)
    small = _layer(2, 300, 1024, 0, 3, 64, 3, torch.float32)
    for rep in range(2):
        w1, g1 = _both(big, 256, 256)
        assert torch.isfinite(w1).all() and torch.equal(w1, g1)
        w2, g2 = _both(small, 0, 64)
        assert torch.isfinite(w2).all() and torch.equal(w2, g2)


def test_static_scratch_forward_refuses_what_does_not_fit():
    limit = ptq.ptq_lopro_linear_forward_static_limit()
    assert limit == 32 << 20
    m, n, tokens = 16384, 16384, 8
    from paper_2601_19675_amd import binding
    assert ptq.ptq_workspace_bytes(binding.OP_LINEAR_FORWARD, m, n, tokens, 0) > limit
    L = _layer(3, 64, 1024, 0, 4, 128, tokens, torch.float32)
    lib = ptq.load_library()
    O = torch.empty((tokens, m), dtype=torch.float32, device="cuda")
    # the size check comes before anything is read: the (small) buffers are never touched
    rc = lib.ptq_lopro_linear_forward_static(L["X"].data_ptr(), 0, n, tokens, m, n, L["packed"].data_ptr(), 4,
                                             L["st"].data_ptr(), L["zt"].data_ptr(), 128, L["perm"].data_ptr(), 0, 64,
                                             None, None, None, 0, None, O.data_ptr(), m, None)
    assert rc == 4   # PTQ_ERR_WORKSPACE
