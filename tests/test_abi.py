"""Host-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and turns bad arguments into status codes before touching a
GPU (none of these calls reaches a kernel launch)."""
import ctypes
import os
import re

import pytest

import paper_2601_19675_amd as ptq
from paper_2601_19675_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ptq.lib_path()):
        from paper_2601_19675_amd import build
        build.build(verbose=False)
    return ptq.load_library()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "ptq.h")).read()
    names = sorted(set(re.findall(r"\b(ptq_[a-z_]+)\s*\(", header)))
    assert {"ptq_hessian_accumulate", "ptq_damped_cholesky_inv", "ptq_quantize_layer",
            "ptq_layer_error", "ptq_workspace_bytes", "ptq_status_string"} <= set(names)
    for nm in names:
        assert hasattr(lib, nm), nm


def test_status_strings_and_workspace_sizes(lib):
    assert ptq.ptq_status_string(0) == "ok"
    assert "positive definite" in ptq.ptq_status_string(5)
    for op in range(9):
        assert ptq.ptq_workspace_bytes(op, 4096, 4096, 262144, 128) % 256 == 0
    # the factorization works on one n x n float64 copy
    assert ptq.ptq_workspace_bytes(binding.OP_CHOLESKY_INV, 0, 4096) >= 4096 * 4096 * 8
    # the solve keeps the errors of every column: n x m float64
    assert ptq.ptq_workspace_bytes(binding.OP_QUANTIZE, 4096, 11008) >= 4096 * 11008 * 8
    # the layer error: room for either form -- float64 copies of D and W, or bfloat16 pieces of D, W and
    # the transposed Hessian on sizes rounded up to its 128-wide tiles
    for mm, nn in ((4096, 4096), (4096, 11008), (1, 1), (70, 200)):
        need = ptq.ptq_workspace_bytes(binding.OP_LAYER_ERROR, mm, nn)
        mp, npad = -(-mm // 128) * 128, -(-nn // 128) * 128
        assert need >= 2 * mm * nn * 8
        assert need >= 2 * 3 * mp * npad * 2 + 3 * npad * npad * 2
    out = ctypes.c_size_t()
    assert lib.ptq_workspace_bytes(0, -1, 8, 8, 0, ctypes.byref(out)) == 2
    assert lib.ptq_workspace_bytes(9, 1, 8, 8, 0, ctypes.byref(out)) == 1
    assert lib.ptq_workspace_bytes(0, 1, 8, 8, 0, None) == 1


def test_argument_errors_are_reported_on_the_host(lib):
    p = 0x1000  # never dereferenced: every call below fails validation first
    # Hessian
    assert lib.ptq_hessian_accumulate(p, 8, p, 1, 16, 16, 8, p, 1 << 20, None) == 2   # ldx < n
    assert lib.ptq_hessian_accumulate(p, 16, p, 2, 16, 16, 16, p, 1 << 20, None) == 3  # f64 X
    assert lib.ptq_hessian_accumulate(p, 12, p, 1, 16, 12, 12, p, 1 << 20, None) == 2  # bf16 n % 8
    assert lib.ptq_hessian_accumulate(None, 16, p, 1, 16, 16, 16, p, 1 << 20, None) == 1
    assert lib.ptq_hessian_accumulate(p, 16, p, 1, 16, 16, 16, None, 0, None) == 4
    assert lib.ptq_hessian_accumulate(p, 16, p, 1, 0, 16, 16, None, 0, None) == 0      # t == 0: no-op
    # factor
    assert lib.ptq_damped_cholesky_inv(p, 16, 16, -0.5, p, 16, None, p, p, 1 << 20, None) == 1
    assert lib.ptq_damped_cholesky_inv(p, 16, 16, float("nan"), p, 16, None, p, p, 1 << 20, None) == 1
    assert lib.ptq_damped_cholesky_inv(p, 8, 16, 0.01, p, 16, None, p, p, 1 << 20, None) == 2
    assert lib.ptq_damped_cholesky_inv(p, 16, 16, 0.01, p, 16, None, None, p, 1 << 20, None) == 1
    assert lib.ptq_damped_cholesky_inv(p, 16, 16, 0.01, p, 16, None, p, p, 16, None) == 4
    # solve
    def q(bits=4, group=16, block=16, n=32, ldw=32, ws=1 << 20, wdt=1):
        return lib.ptq_quantize_layer(p, wdt, ldw, 4, n, p, n, None, bits, group, block, p, p, p, None, None,
                                      p, ws, None)
    assert q(bits=1) == 1 and q(bits=9) == 1
    assert q(wdt=9) == 3
    assert q(group=12) == 2            # n % group
    assert q(group=8, block=16) == 2   # groups start on 16-column boundaries
    assert q(block=24) == 2 and q(block=512, group=16, n=1024, ldw=1024) == 2
    assert q(group=32, block=48, n=96, ldw=96) == 2   # neither divides the other
    assert q(ldw=16) == 2
    assert q(ws=64) == 4
    # layer error
    assert lib.ptq_layer_error(p, 1, 32, p, 4, 32, p, 16, p, p, 1 << 20, None) == 2   # ldh < n
    assert lib.ptq_layer_error(p, 1, 32, None, 4, 32, p, 32, p, p, 1 << 20, None) == 1
    assert lib.ptq_layer_error(p, 1, 32, p, 0, 32, p, 32, p, p, 1 << 20, None) == 2


def test_lopro_argument_errors_are_reported_on_the_host(lib):
    p = 0x1000  # 32-byte aligned, never dereferenced
    big = 1 << 30
    # rotation shape rules: b_H a power of two in [16, 256], b_I % 4 == 0, (n - b_I) % b_H == 0
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 256, 96, p, 512, None) == 2    # b_H not a power of two
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 256, 512, p, 512, None) == 2   # b_H > 256
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 250, 64, p, 512, None) == 2    # b_I % 4
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 128, 256, p, 512, None) == 2   # (n - b_I) % b_H
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 256, 256, p, 510, None) == 2   # ldo
    assert lib.ptq_lopro_rotate_weight(p, 5, 512, 4, 512, p, 256, 256, p, 512, None) == 3   # dtype
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, None, 256, 256, p, 512, None) == 1
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 4, 512, p, 256, 256, p + 8, 512, None) == 1  # misaligned output
    assert lib.ptq_lopro_rotate_weight(p, 1, 512, 0, 512, p, 256, 256, p, 512, None) == 0   # m == 0: no-op
    assert lib.ptq_lopro_unrotate_weight(p, 512, 4, 512, p, 256, 256, p, 512, None) == 1    # in place
    assert lib.ptq_lopro_unrotate_weight(p, 510, 4, 512, p, 256, 256, p + 64, 512, None) == 2
    assert lib.ptq_lopro_rotate_hessian(p, 512, 512, p, 256, 256, p + 64, 512, None, 0, None) == 4
    assert lib.ptq_lopro_rotate_hessian(p, 512, 512, p, 256, 256, p, 512, p, big, None) == 1   # in place
    assert lib.ptq_lopro_rotate_hessian(p, 256, 512, p, 256, 256, p + 64, 512, p, big, None) == 2
    assert lib.ptq_lopro_column_order(p, 1, 512, 4, 512, p, 512, 1, p, None, None, 0, None) == 4
    assert lib.ptq_lopro_column_order(p, 1, 256, 4, 512, p, 512, 1, p, None, p, big, None) == 2
    assert lib.ptq_lopro_column_order(p, 1, 512, 4, 512, p, 512, 1, None, None, p, big, None) == 1
    assert lib.ptq_lopro_column_order(p, 1, 512, 0, 512, p, 512, 1, p, None, p, big, None) == 2  # no rows: keys undefined


def test_low_rank_step_argument_errors_are_reported_on_the_host(lib):
    p = 0x1000
    big = 1 << 34
    # activation sums
    assert lib.ptq_activation_abs_sum(p, p, 2, 16, 16, 16, p, big, None) == 3        # f64 X
    assert lib.ptq_activation_abs_sum(p, p, 1, 16, 12, 16, p, big, None) == 2        # n % 8
    assert lib.ptq_activation_abs_sum(p, p, 1, 16, 16, 8, p, big, None) == 2         # ldx < n
    assert lib.ptq_activation_abs_sum(None, p, 1, 16, 16, 16, p, big, None) == 1
    assert lib.ptq_activation_abs_sum(p, p + 2, 1, 16, 16, 16, p, big, None) == 1    # misaligned X
    assert lib.ptq_activation_abs_sum(p, p, 1, 16, 16, 16, None, 0, None) == 4
    assert lib.ptq_activation_abs_sum(p, p, 1, 0, 16, 16, None, 0, None) == 0        # no tokens: no-op
    assert lib.ptq_activation_scale(p, 0, 16, p, None) == 2                          # tokens must be positive
    assert lib.ptq_activation_scale(None, 4, 16, p, None) == 1
    # the sketch:              W  dt ldw  m   n   s  S  lds r  it U  V  sg R  ldr ws  bytes
    ok = (p, 0, 64, 8, 64, p, p, 64, 2, 2, p, p, p, p + 64, 64, p, big, None)
    def call(**kw):
        a = list(ok)
        names = ["W", "dt", "ldw", "m", "n", "s", "S", "lds", "r", "it", "U", "V", "sg", "R", "ldr", "ws", "bytes"]
        for k, v in kw.items():
            a[names.index(k)] = v
        return lib.ptq_scaled_r1svd(*a)
    assert call(dt=7) == 3
    assert call(n=62, ldw=62, ldr=64) == 2           # n % 4
    assert call(ldr=66) == 2                         # ldr % 4
    assert call(ldw=32) == 2
    assert call(lds=32) == 2
    assert call(lds=66) == 2                         # lds % 4
    assert call(S=p + 4) == 1                        # misaligned sketch vectors
    assert call(n=32772, ldw=32772, ldr=32772, lds=32772) == 2   # more columns than the kernels hold
    assert call(r=-1) == 1
    assert call(it=-1) == 1
    assert call(S=None) == 1
    assert call(R=p) == 1                            # in place
    assert call(R=p + 4) == 1                        # misaligned
    assert call(ws=None, bytes=0) == 4
    assert call(bytes=1024) == 4


def test_stored_form_argument_errors_and_average_bits(lib):
    p = 0x1000
    big = 1 << 34
    # Eq. 12 on the host: 2 bits, group 128, 16-bit originals, rank 16 in 8 bits, 4096 x 4096
    want = 2 + 16 / 128 + 2 * (16 * 8 / 4096) + 2 * 16 / 4096 + 16 * 16 / 4096 ** 2
    assert abs(ptq.ptq_average_bits(4096, 4096, 2, 16, 128, 16, 8) - want) < 1e-15
    assert ptq.ptq_average_bits(0, 4096, 2, 16, 128, 16, 8) == -1.0
    # packing
    g0 = (None, None, 0, None, None, None)                                # codes only
    assert lib.ptq_pack_codes(p, 64, 4, 64, 5, p, *g0) == 1          # bits
    assert lib.ptq_pack_codes(p, 64, 4, 48, 4, p, *g0) == 2          # n % 32
    assert lib.ptq_pack_codes(p, 72, 4, 64, 4, p, *g0) == 2          # ldc % 16
    assert lib.ptq_pack_codes(p + 8, 64, 4, 64, 4, p, *g0) == 1      # misaligned codes
    assert lib.ptq_pack_codes(None, 64, 4, 64, 4, p, *g0) == 1
    assert lib.ptq_pack_codes(p, 64, 0, 64, 4, p, *g0) == 0
    assert lib.ptq_pack_codes(p, 64, 4, 64, 4, p, p, p, 48, p + 64, p + 128, None) == 2   # n % group
    assert lib.ptq_pack_codes(p, 64, 4, 64, 4, p, p, p, 32, None, p + 128, None) == 1    # grids: all or none
    assert lib.ptq_pack_codes(p, 64, 4, 64, 4, p, p, p, 32, p, p + 128, None) == 1       # in place
    assert lib.ptq_unpack_dequantize(p, 4, 64, 4, p, p, 48, p, 64, None) == 2   # n % group
    assert lib.ptq_unpack_dequantize(p, 4, 64, 4, p, p, 32, p, 32, None) == 2   # ldq < n
    assert lib.ptq_unpack_dequantize(p, 4, 64, 4, None, p, 32, p, 64, None) == 1
    # vector quantizer:          W dt ldw m  n   U ldu dead cb  K   d blk idx Wq e2 ws bytes
    vq = lambda **kw: lib.ptq_quantize_layer_vq(*[kw.get(k, v) for k, v in dict(
        W=p, dt=1, ldw=64, m=8, n=64, U=p, ldu=64, dead=None, cb=p, K=256, d=4, blk=64, idx=p, Wq=None, e2=None, ws=p,
        bytes=big, st=None).items()])
    assert vq(K=0) == 1 and vq(K=257) == 1 and vq(d=3) == 1 and vq(dt=7) == 3
    assert vq(n=62, ldw=62, ldu=62) == 2 and vq(blk=40) == 2 and vq(blk=512) == 2 and vq(ldu=32) == 2
    assert vq(cb=None) == 1 and vq(idx=None) == 1 and vq(ws=None, bytes=0) == 4 and vq(m=0) == 0
    # forward:                  X  dt ldx tok m  n    packed bits sc z  grp perm bI  bH  U  V  sg r  s  O  ldo ws bytes
    ok = [p, 0, 256, 2, 8, 256, p, 4, p, p, 64, p, 128, 128, p, p, p, 4, p, p, 8, p, big, None]
    names = ["X", "dt", "ldx", "tok", "m", "n", "packed", "bits", "sc", "z", "grp", "perm", "bI", "bH", "U", "V",
             "sg", "r", "s", "O", "ldo", "ws", "bytes"]
    def call(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return lib.ptq_lopro_linear_forward(*a)
    assert call(dt=9) == 3
    assert call(bits=5) == 1
    assert call(grp=48) == 2                     # group % 32
    assert call(ldo=4) == 2
    assert call(ldx=128) == 2
    assert call(bH=96) == 2                      # rotation shape rules
    assert call(tok=5000) == 2
    assert call(U=None) == 1
    assert call(perm=None) == 1
    assert call(ws=None, bytes=0) == 4
    assert call(tok=0) == 0
    # the form on the library's own scratch array: the same checks, and sizes beyond the array are refused
    def call_static(**kw):
        a = list(ok)
        for k, v in kw.items():
            a[names.index(k)] = v
        return lib.ptq_lopro_linear_forward_static(*(a[:21] + [None]))
    assert call_static(dt=9) == 3 and call_static(bits=5) == 1 and call_static(grp=48) == 2
    assert call_static(U=None) == 1 and call_static(tok=0) == 0
    assert lib.ptq_lopro_linear_forward_static_limit() == 32 << 20
    assert ptq.ptq_workspace_bytes(binding.OP_LINEAR_FORWARD, 16384, 16384, 8, 4) > 32 << 20
    assert call_static(m=16384, n=16384, ldx=16384, ldo=16384, tok=8) == 4
