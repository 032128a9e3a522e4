"""Thin ctypes binding of libptq's C ABI (include/ptq.h).

Argument marshalling only: every function takes torch tensors that already
live on the GPU (torch is used for device memory and streams, nothing else),
passes their raw pointers, sizes and the current HIP stream to the entry point
of the same name, and raises PtqError on a non-zero status.  There is no CPU
or PyTorch fallback: without the built library every call fails loudly.
"""
from __future__ import annotations

import ctypes
import os

import torch

PTQ_F32, PTQ_BF16, PTQ_F64 = 0, 1, 2
OP_HESSIAN, OP_CHOLESKY_INV, OP_QUANTIZE, OP_LAYER_ERROR = 0, 1, 2, 3
OP_LOPRO_ORDER, OP_LOPRO_ROTATE_HESSIAN = 4, 5
OP_ACTIVATION_ABS_SUM, OP_SCALED_R1SVD, OP_LINEAR_FORWARD = 6, 7, 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class PtqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {ptq_status_string(status)} (status {status})")


def lib_path() -> str:
    return os.path.join(_HERE, "libptq.so")


def load_library() -> ctypes.CDLL:
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it with `python -m paper_2601_19675_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    c = ctypes
    i64, vp, sz = c.c_int64, c.c_void_p, c.c_size_t
    lib.ptq_status_string.restype = c.c_char_p
    lib.ptq_status_string.argtypes = [c.c_int]
    lib.ptq_workspace_bytes.restype = c.c_int
    lib.ptq_workspace_bytes.argtypes = [c.c_int, i64, i64, i64, i64, c.POINTER(sz)]
    lib.ptq_hessian_accumulate.restype = c.c_int
    lib.ptq_hessian_accumulate.argtypes = [vp, i64, vp, c.c_int, i64, i64, i64, vp, sz, vp]
    lib.ptq_damped_cholesky_inv.restype = c.c_int
    lib.ptq_damped_cholesky_inv.argtypes = [vp, i64, i64, c.c_double, vp, i64, vp, vp, vp, sz, vp]
    for fn in (lib.ptq_quantize_layer, lib.ptq_quantize_layer_static_groups):
        fn.restype = c.c_int
        fn.argtypes = [vp, c.c_int, i64, i64, i64, vp, i64, vp, c.c_int, c.c_int, c.c_int, vp, vp, vp, vp, vp, vp,
                       sz, vp]
    lib.ptq_quantize_layer_vq.restype = c.c_int
    lib.ptq_quantize_layer_vq.argtypes = [vp, c.c_int, i64, i64, i64, vp, i64, vp, vp, c.c_int, c.c_int, c.c_int, vp, vp,
                                          vp, vp, sz, vp]
    lib.ptq_layer_error.restype = c.c_int
    lib.ptq_layer_error.argtypes = [vp, c.c_int, i64, vp, i64, i64, vp, i64, vp, vp, sz, vp]
    lib.ptq_lopro_column_order.restype = c.c_int
    lib.ptq_lopro_column_order.argtypes = [vp, c.c_int, i64, i64, i64, vp, i64, c.c_int, vp, vp, vp, sz, vp]
    lib.ptq_lopro_rotate_weight.restype = c.c_int
    lib.ptq_lopro_rotate_weight.argtypes = [vp, c.c_int, i64, i64, i64, vp, c.c_int, c.c_int, vp, i64, vp]
    lib.ptq_lopro_unrotate_weight.restype = c.c_int
    lib.ptq_lopro_unrotate_weight.argtypes = [vp, i64, i64, i64, vp, c.c_int, c.c_int, vp, i64, vp]
    lib.ptq_lopro_rotate_hessian.restype = c.c_int
    lib.ptq_lopro_rotate_hessian.argtypes = [vp, i64, i64, vp, c.c_int, c.c_int, vp, i64, vp, sz, vp]
    lib.ptq_activation_abs_sum.restype = c.c_int
    lib.ptq_activation_abs_sum.argtypes = [vp, vp, c.c_int, i64, i64, i64, vp, sz, vp]
    lib.ptq_activation_scale.restype = c.c_int
    lib.ptq_activation_scale.argtypes = [vp, i64, i64, vp, vp]
    lib.ptq_average_bits.restype = c.c_double
    lib.ptq_average_bits.argtypes = [i64, i64, c.c_double, c.c_double, i64, i64, c.c_double]
    lib.ptq_pack_codes.restype = c.c_int
    lib.ptq_pack_codes.argtypes = [vp, i64, i64, i64, c.c_int, vp, vp, vp, c.c_int, vp, vp, vp]
    lib.ptq_unpack_dequantize.restype = c.c_int
    lib.ptq_unpack_dequantize.argtypes = [vp, i64, i64, c.c_int, vp, vp, c.c_int, vp, i64, vp]
    lib.ptq_lopro_linear_forward.restype = c.c_int
    lib.ptq_lopro_linear_forward.argtypes = [vp, c.c_int, i64, i64, i64, i64, vp, c.c_int, vp, vp, c.c_int, vp,
                                             c.c_int, c.c_int, vp, vp, vp, c.c_int, vp, vp, i64, vp, sz, vp]
    lib.ptq_lopro_linear_forward_static.restype = c.c_int
    lib.ptq_lopro_linear_forward_static.argtypes = lib.ptq_lopro_linear_forward.argtypes[:21] + [vp]
    lib.ptq_lopro_linear_forward_static_limit.restype = sz
    lib.ptq_lopro_linear_forward_static_limit.argtypes = []
    lib.ptq_scaled_r1svd.restype = c.c_int
    lib.ptq_scaled_r1svd.argtypes = [vp, c.c_int, i64, i64, i64, vp, vp, i64, c.c_int, c.c_int, vp, vp, vp, vp,
                                     i64, vp, sz, vp]
    _LIB = lib
    return lib


def ptq_status_string(status: int) -> str:
    return load_library().ptq_status_string(int(status)).decode()


def ptq_workspace_bytes(op: int, m: int = 0, n: int = 0, t: int = 0, block: int = 0) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().ptq_workspace_bytes(op, m, n, t, block, ctypes.byref(out))
    if rc:
        raise PtqError(rc, "ptq_workspace_bytes")
    return int(out.value)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PTQ_F32
    if t.dtype == torch.bfloat16:
        return PTQ_BF16
    if t.dtype == torch.float64:
        return PTQ_F64
    raise PtqError(3, f"tensor dtype {t.dtype}")


def _check_dev(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda):
            raise ValueError("libptq takes device tensors only")


def _ws(ws: torch.Tensor | None, need: int, like: torch.Tensor) -> torch.Tensor:
    if ws is None:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=like.device)
    return ws


def ptq_hessian_accumulate(H: torch.Tensor, X: torch.Tensor, ws: torch.Tensor | None = None) -> None:
    """H[upper] += X^T X.  H: n x n float64; X: t x n bfloat16 or float32."""
    _check_dev(H, X)
    t, n = X.shape
    assert H.dtype == torch.float64 and H.shape == (n, n) and H.stride(1) == 1 and X.stride(1) == 1
    ws = _ws(ws, ptq_workspace_bytes(OP_HESSIAN, 0, n, t), H)
    rc = load_library().ptq_hessian_accumulate(H.data_ptr(), H.stride(0), X.data_ptr(), _dtype_code(X), t,
                                               n, X.stride(0), ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_hessian_accumulate")


def ptq_damped_cholesky_inv(H: torch.Tensor, damp: float, U: torch.Tensor,
                            dead_mask: torch.Tensor | None, info: torch.Tensor,
                            ws: torch.Tensor | None = None) -> None:
    """U <- upper factor with U^T U = (H' + damp mean(diag H') I)^-1; info: int32[2] on device."""
    _check_dev(H, U, dead_mask, info)
    n = H.shape[0]
    assert H.dtype == torch.float64 and U.dtype == torch.float64 and info.dtype == torch.int32
    assert H.stride(1) == 1 and U.stride(1) == 1 and U.shape == (n, n) and info.numel() >= 2
    assert dead_mask is None or (dead_mask.dtype == torch.uint8 and dead_mask.numel() >= n)
    ws = _ws(ws, ptq_workspace_bytes(OP_CHOLESKY_INV, 0, n), H)
    rc = load_library().ptq_damped_cholesky_inv(H.data_ptr(), H.stride(0), n, float(damp), U.data_ptr(),
                                                U.stride(0), _ptr(dead_mask), info.data_ptr(),
                                                ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_damped_cholesky_inv")


def ptq_quantize_layer(W: torch.Tensor, U: torch.Tensor, dead_mask: torch.Tensor | None, bits: int,
                       group: int, block: int, codes: torch.Tensor, scales: torch.Tensor,
                       zeros: torch.Tensor, Wq: torch.Tensor | None = None,
                       row_err2: torch.Tensor | None = None, ws: torch.Tensor | None = None,
                       _entry: str = "ptq_quantize_layer") -> None:
    """Column-sequential quantize + compensate of W (m x n) with factor U."""
    _check_dev(W, U, dead_mask, codes, scales, zeros, Wq, row_err2)
    m, n = W.shape
    assert W.stride(1) == 1 and U.stride(1) == 1 and U.dtype == torch.float64
    assert codes.dtype == torch.uint8 and codes.is_contiguous() and codes.shape == (m, n)
    if group > 0 and n % group == 0:
        assert scales.dtype == torch.float32 and scales.is_contiguous() and scales.shape == (m, n // group)
        assert zeros.dtype == torch.uint8 and zeros.is_contiguous() and zeros.shape == (m, n // group)
    assert Wq is None or (Wq.dtype == torch.float64 and Wq.is_contiguous() and Wq.shape == (m, n))
    assert row_err2 is None or (row_err2.dtype == torch.float64 and row_err2.numel() >= m)
    ws = _ws(ws, ptq_workspace_bytes(OP_QUANTIZE, m, n), W)
    rc = getattr(load_library(), _entry)(W.data_ptr(), _dtype_code(W), W.stride(0), m, n, U.data_ptr(),
                                         U.stride(0), _ptr(dead_mask), bits, group, block,
                                         codes.data_ptr(), scales.data_ptr(), zeros.data_ptr(), _ptr(Wq),
                                         _ptr(row_err2), ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, _entry)


def ptq_quantize_layer_static_groups(W: torch.Tensor, U: torch.Tensor, dead_mask: torch.Tensor | None, bits: int,
                                     group: int, block: int, codes: torch.Tensor, scales: torch.Tensor,
                                     zeros: torch.Tensor, Wq: torch.Tensor | None = None,
                                     row_err2: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> None:
    """The same solve with every group's grid taken from W as given, before any compensation."""
    ptq_quantize_layer(W, U, dead_mask, bits, group, block, codes, scales, zeros, Wq, row_err2, ws,
                       _entry="ptq_quantize_layer_static_groups")


def ptq_quantize_layer_vq(W: torch.Tensor, U: torch.Tensor, dead_mask: torch.Tensor | None, codebook: torch.Tensor,
                          block: int, indices: torch.Tensor, Wq: torch.Tensor | None = None,
                          row_err2: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> None:
    """The column solve with a vector quantizer: codebook (float32 entries x dim), indices (uint8 m x n/dim)."""
    _check_dev(W, U, dead_mask, codebook, indices, Wq, row_err2)
    m, n = W.shape
    entries, dim = codebook.shape
    assert W.stride(1) == 1 and U.stride(1) == 1 and U.dtype == torch.float64
    assert codebook.dtype == torch.float32 and codebook.is_contiguous()
    if dim > 0 and n % dim == 0:
        assert indices.dtype == torch.uint8 and indices.is_contiguous() and indices.shape == (m, n // dim)
    assert Wq is None or (Wq.dtype == torch.float64 and Wq.is_contiguous() and Wq.shape == (m, n))
    assert row_err2 is None or (row_err2.dtype == torch.float64 and row_err2.numel() >= m)
    ws = _ws(ws, ptq_workspace_bytes(OP_QUANTIZE, m, n), W)
    rc = load_library().ptq_quantize_layer_vq(W.data_ptr(), _dtype_code(W), W.stride(0), m, n, U.data_ptr(), U.stride(0),
                                              _ptr(dead_mask), codebook.data_ptr(), entries, dim, block,
                                              indices.data_ptr(), _ptr(Wq), _ptr(row_err2), ws.data_ptr(), ws.numel(),
                                              _stream())
    if rc:
        raise PtqError(rc, "ptq_quantize_layer_vq")


def ptq_layer_error(W: torch.Tensor, Wq: torch.Tensor, H: torch.Tensor, out: torch.Tensor,
                    ws: torch.Tensor | None = None) -> None:
    """out[0:3] <- (rel, num, den) of the proxy-Hessian layer error."""
    _check_dev(W, Wq, H, out)
    m, n = W.shape
    assert Wq.dtype == torch.float64 and Wq.is_contiguous() and Wq.shape == (m, n)
    assert H.dtype == torch.float64 and H.stride(1) == 1 and out.dtype == torch.float64 and out.numel() >= 3
    ws = _ws(ws, ptq_workspace_bytes(OP_LAYER_ERROR, m, n), W)
    rc = load_library().ptq_layer_error(W.data_ptr(), _dtype_code(W), W.stride(0), Wq.data_ptr(), m, n,
                                        H.data_ptr(), H.stride(0), out.data_ptr(), ws.data_ptr(),
                                        ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_layer_error")


def ptq_lopro_column_order(R: torch.Tensor, H: torch.Tensor, perm: torch.Tensor, descending: bool = True,
                           keys: torch.Tensor | None = None, ws: torch.Tensor | None = None) -> None:
    """perm <- columns ordered by diag(H) / mean|R| (int32[n]); keys (float64[n]) optional."""
    _check_dev(R, H, perm, keys)
    m, n = R.shape
    assert R.stride(1) == 1 and H.dtype == torch.float64 and H.stride(1) == 1
    assert perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() >= n
    assert keys is None or (keys.dtype == torch.float64 and keys.is_contiguous() and keys.numel() >= n)
    ws = _ws(ws, ptq_workspace_bytes(OP_LOPRO_ORDER, m, n), R)
    rc = load_library().ptq_lopro_column_order(R.data_ptr(), _dtype_code(R), R.stride(0), m, n, H.data_ptr(),
                                               H.stride(0), int(bool(descending)), perm.data_ptr(),
                                               _ptr(keys), ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_lopro_column_order")


def ptq_lopro_rotate_weight(R: torch.Tensor, perm: torch.Tensor, b_I: int, b_H: int, Rout: torch.Tensor) -> None:
    """Rout <- R P Q (float64)."""
    _check_dev(R, perm, Rout)
    m, n = R.shape
    assert R.stride(1) == 1 and perm.dtype == torch.int32 and perm.is_contiguous()
    assert Rout.dtype == torch.float64 and Rout.stride(1) == 1 and Rout.shape == (m, n)
    rc = load_library().ptq_lopro_rotate_weight(R.data_ptr(), _dtype_code(R), R.stride(0), m, n, perm.data_ptr(),
                                                b_I, b_H, Rout.data_ptr(), Rout.stride(0), _stream())
    if rc:
        raise PtqError(rc, "ptq_lopro_rotate_weight")


def ptq_lopro_unrotate_weight(Rq: torch.Tensor, perm: torch.Tensor, b_I: int, b_H: int, Wout: torch.Tensor) -> None:
    """Wout <- Rq Q^T P^T (float64)."""
    _check_dev(Rq, perm, Wout)
    m, n = Rq.shape
    assert Rq.dtype == torch.float64 and Rq.stride(1) == 1 and perm.dtype == torch.int32 and perm.is_contiguous()
    assert Wout.dtype == torch.float64 and Wout.stride(1) == 1 and Wout.shape == (m, n)
    rc = load_library().ptq_lopro_unrotate_weight(Rq.data_ptr(), Rq.stride(0), m, n, perm.data_ptr(), b_I, b_H,
                                                  Wout.data_ptr(), Wout.stride(0), _stream())
    if rc:
        raise PtqError(rc, "ptq_lopro_unrotate_weight")


def ptq_lopro_rotate_hessian(H: torch.Tensor, perm: torch.Tensor, b_I: int, b_H: int, Hout: torch.Tensor,
                             ws: torch.Tensor | None = None) -> None:
    """Hout <- Q^T P^T H P Q (full symmetric, float64); only H's upper triangle is read."""
    _check_dev(H, perm, Hout)
    n = H.shape[0]
    assert H.dtype == torch.float64 and H.stride(1) == 1 and perm.dtype == torch.int32 and perm.is_contiguous()
    assert Hout.dtype == torch.float64 and Hout.stride(1) == 1 and Hout.shape == (n, n)
    ws = _ws(ws, ptq_workspace_bytes(OP_LOPRO_ROTATE_HESSIAN, 0, n), H)
    rc = load_library().ptq_lopro_rotate_hessian(H.data_ptr(), H.stride(0), n, perm.data_ptr(), b_I, b_H,
                                                 Hout.data_ptr(), Hout.stride(0), ws.data_ptr(), ws.numel(),
                                                 _stream())
    if rc:
        raise PtqError(rc, "ptq_lopro_rotate_hessian")


def ptq_activation_abs_sum(asum: torch.Tensor, X: torch.Tensor, ws: torch.Tensor | None = None) -> None:
    """asum[j] += sum_k |X[k, j]| (float64[n], accumulated in place)."""
    _check_dev(asum, X)
    t, n = X.shape
    assert X.stride(1) == 1 and asum.dtype == torch.float64 and asum.is_contiguous() and asum.numel() >= n
    ws = _ws(ws, ptq_workspace_bytes(OP_ACTIVATION_ABS_SUM, 0, n), X)
    rc = load_library().ptq_activation_abs_sum(asum.data_ptr(), X.data_ptr(), _dtype_code(X), t, n, X.stride(0),
                                               ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_activation_abs_sum")


def ptq_activation_scale(asum: torch.Tensor, tokens: int, s: torch.Tensor) -> None:
    """s <- Xbar^2.5 / sqrt(max(Xbar) min(Xbar)), Xbar = asum / tokens (float64[n])."""
    _check_dev(asum, s)
    n = asum.numel()
    assert asum.dtype == torch.float64 and asum.is_contiguous()
    assert s.dtype == torch.float64 and s.is_contiguous() and s.numel() >= n
    rc = load_library().ptq_activation_scale(asum.data_ptr(), int(tokens), n, s.data_ptr(), _stream())
    if rc:
        raise PtqError(rc, "ptq_activation_scale")


def ptq_scaled_r1svd(W: torch.Tensor, s: torch.Tensor, S: torch.Tensor, it: int, U: torch.Tensor, V: torch.Tensor,
                     sigma: torch.Tensor, R: torch.Tensor, ws: torch.Tensor | None = None) -> None:
    """Rank-by-rank sketch of W diag(s): U (uint8 r x m), V (uint8 r x n) e4m3 codes, sigma (float16 r),
    R (float32 m x n) the residual; S (float32 r x n) holds the random vector of each rank."""
    _check_dev(W, s, S, U, V, sigma, R)
    m, n = W.shape
    r = S.shape[0]
    assert W.stride(1) == 1 and s.dtype == torch.float64 and s.is_contiguous() and s.numel() == n
    assert S.dtype == torch.float32 and S.shape == (r, n) and (r == 0 or S.stride(1) == 1)
    assert U.dtype == torch.uint8 and U.is_contiguous() and U.shape == (r, m)
    assert V.dtype == torch.uint8 and V.is_contiguous() and V.shape == (r, n)
    assert sigma.dtype == torch.float16 and sigma.is_contiguous() and sigma.numel() == r
    assert R.dtype == torch.float32 and R.stride(1) == 1 and R.shape == (m, n)
    ws = _ws(ws, ptq_workspace_bytes(OP_SCALED_R1SVD, m, n), W)
    rc = load_library().ptq_scaled_r1svd(W.data_ptr(), _dtype_code(W), W.stride(0), m, n, s.data_ptr(),
                                         S.data_ptr(), S.stride(0) if r else n, r, int(it), U.data_ptr(),
                                         V.data_ptr(), sigma.data_ptr(), R.data_ptr(), R.stride(0),
                                         ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_scaled_r1svd")


def ptq_average_bits(m: int, n: int, d_q: float, d_o: float, g: int, r: int, d_r: float) -> float:
    """Eq. 12: average bits per weight of a stored layer (host arithmetic)."""
    return float(load_library().ptq_average_bits(m, n, d_q, d_o, g, r, d_r))


def ptq_pack_codes(codes: torch.Tensor, bits: int, packed: torch.Tensor, scales: torch.Tensor | None = None,
                   zeros: torch.Tensor | None = None, group: int = 0, scales_t: torch.Tensor | None = None,
                   zeros_t: torch.Tensor | None = None) -> None:
    """packed (int32 n/32 x m x bits, chunk-major) <- bit stream of codes (uint8 m x n); with the grids given,
    scales_t / zeros_t (n/group x m) <- scales / zeros (m x n/group)."""
    _check_dev(codes, packed, scales, zeros, scales_t, zeros_t)
    m, n = codes.shape
    assert codes.dtype == torch.uint8 and codes.stride(1) == 1
    assert packed.dtype == torch.int32 and packed.is_contiguous() and packed.shape == (n // 32, m, bits)
    if scales is not None:
        ng = n // group
        assert scales.dtype == torch.float32 and scales.is_contiguous() and scales.shape == (m, ng)
        assert zeros.dtype == torch.uint8 and zeros.is_contiguous() and zeros.shape == (m, ng)
        assert scales_t.dtype == torch.float32 and scales_t.is_contiguous() and scales_t.shape == (ng, m)
        assert zeros_t.dtype == torch.uint8 and zeros_t.is_contiguous() and zeros_t.shape == (ng, m)
    rc = load_library().ptq_pack_codes(codes.data_ptr(), codes.stride(0), m, n, bits, packed.data_ptr(), _ptr(scales),
                                       _ptr(zeros), group, _ptr(scales_t), _ptr(zeros_t), _stream())
    if rc:
        raise PtqError(rc, "ptq_pack_codes")


def ptq_unpack_dequantize(packed: torch.Tensor, n: int, bits: int, scales_t: torch.Tensor, zeros_t: torch.Tensor,
                          group: int, Wq: torch.Tensor) -> None:
    """Wq (float64 m x n) <- scale * (code - zero) from the packed codes and group-major grids."""
    _check_dev(packed, scales_t, zeros_t, Wq)
    m = packed.shape[1]
    assert packed.dtype == torch.int32 and packed.is_contiguous() and packed.shape == (n // 32, m, bits)
    assert scales_t.dtype == torch.float32 and scales_t.is_contiguous() and scales_t.shape == (n // group, m)
    assert zeros_t.dtype == torch.uint8 and zeros_t.is_contiguous() and zeros_t.shape == (n // group, m)
    assert Wq.dtype == torch.float64 and Wq.stride(1) == 1 and Wq.shape == (m, n)
    rc = load_library().ptq_unpack_dequantize(packed.data_ptr(), m, n, bits, scales_t.data_ptr(), zeros_t.data_ptr(),
                                              group, Wq.data_ptr(), Wq.stride(0), _stream())
    if rc:
        raise PtqError(rc, "ptq_unpack_dequantize")


def ptq_lopro_linear_forward(X: torch.Tensor, packed: torch.Tensor, bits: int, scales_t: torch.Tensor,
                             zeros_t: torch.Tensor, group: int, perm: torch.Tensor, b_I: int, b_H: int,
                             U: torch.Tensor | None, V: torch.Tensor | None, sigma: torch.Tensor | None,
                             s: torch.Tensor | None, O: torch.Tensor, ws: torch.Tensor | None = None,
                             _static: bool = False) -> None:
    """O (float32 tokens x m) <- the stored layer applied to X (tokens x n) in the rotated-input form;
    scales_t / zeros_t are the group-major grids ptq_pack_codes writes."""
    scales, zeros = scales_t, zeros_t
    _check_dev(X, packed, scales, zeros, perm, U, V, sigma, s, O)
    tokens, n = X.shape
    m = packed.shape[1]
    r = 0 if U is None else U.shape[0]
    assert X.stride(1) == 1 and packed.dtype == torch.int32 and packed.is_contiguous()
    assert packed.shape == (n // 32, m, bits)
    assert scales.dtype == torch.float32 and scales.is_contiguous() and scales.shape == (n // group, m)
    assert zeros.dtype == torch.uint8 and zeros.is_contiguous() and zeros.shape == (n // group, m)
    assert perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() == n
    if r:
        assert U.dtype == torch.uint8 and U.is_contiguous() and U.shape == (r, m)
        assert V.dtype == torch.uint8 and V.is_contiguous() and V.shape == (r, n)
        assert sigma.dtype == torch.float16 and sigma.is_contiguous() and sigma.numel() == r
        assert s.dtype == torch.float64 and s.is_contiguous() and s.numel() == n
    assert O.dtype == torch.float32 and O.stride(1) == 1 and O.shape == (tokens, m)
    args = (X.data_ptr(), _dtype_code(X), X.stride(0), tokens, m, n, packed.data_ptr(), bits, scales.data_ptr(),
            zeros.data_ptr(), group, perm.data_ptr(), b_I, b_H, _ptr(U), _ptr(V), _ptr(sigma), r, _ptr(s),
            O.data_ptr(), O.stride(0))
    if _static:
        rc = load_library().ptq_lopro_linear_forward_static(*args, _stream())
        if rc:
            raise PtqError(rc, "ptq_lopro_linear_forward_static")
        return
    ws = _ws(ws, ptq_workspace_bytes(OP_LINEAR_FORWARD, m, n, tokens, r), X)
    rc = load_library().ptq_lopro_linear_forward(*args, ws.data_ptr(), ws.numel(), _stream())
    if rc:
        raise PtqError(rc, "ptq_lopro_linear_forward")


def ptq_lopro_linear_forward_static(X, packed, bits, scales_t, zeros_t, group, perm, b_I, b_H, U, V, sigma, s,
                                    O) -> None:
    """The same call on the library's own per-GPU scratch array: nothing is allocated, no workspace is passed."""
    ptq_lopro_linear_forward(X, packed, bits, scales_t, zeros_t, group, perm, b_I, b_H, U, V, sigma, s, O,
                             _static=True)


def ptq_lopro_linear_forward_static_limit() -> int:
    return int(load_library().ptq_lopro_linear_forward_static_limit())
