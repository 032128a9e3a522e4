"""Why the lazy update of the column solve runs in float64: a CPU emulation of the GPU's blocked scheme in
which only the arithmetic of the update  S = W[:, blk] - E[:, :i1] @ U[:i1, blk]  is swapped for a cheaper
one, held against the oracle by the same near-tie protocol as the GPU.  The rungs: float64; bfloat16 pieces
(4 or 3 per operand) whose products are exact in float32 and are summed in float32 over chunks of 16 or 32
columns and in float64 across chunks; plain float32; three bfloat16 pieces with float32 sums throughout; one
bfloat16 piece.  Every rung below float64 moves the pre-rounding values by 1e-8 .. 1e-7 code steps (1e-3
for bfloat16), which flips the float32 rounding of group scales and near-tie codes in a sizeable share of
the rows -- flagged by the protocol at best, failures at worst -- where float64 flips none.  This test
runs the first configuration (512 x 512, all rows); the same script on 256 sampled rows of the 4096 x 4096
layers and 128 rows of the 4096 x 11008 one gave the table in profiles/lazy_update_precision_ladder.txt."""
import numpy as np
import pytest

import ptq_workloads as wl
from oracle import ptq_oracle as orc
from parity import compare_quantization


def _bf16(a):
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return r.view(np.float32)


def _pieces(a64, k):
    out, rem = [], a64.copy()
    for _ in range(k):
        p = _bf16(rem.astype(np.float32))
        out.append(p)
        rem = rem - p.astype(np.float64)
    return out


def lazy_update(E, U, rung):
    """E @ U in the arithmetic of the rung."""
    if E.shape[1] == 0:
        return np.zeros((E.shape[0], U.shape[1]))
    if rung == "f64":
        return E @ U
    if rung == "f32":
        return (E.astype(np.float32) @ U.astype(np.float32)).astype(np.float64)
    if rung == "bf16":
        return (_bf16(E) @ _bf16(U)).astype(np.float64)
    if rung == "bf16x3":
        ep, up = _pieces(E, 3), _pieces(U, 3)
        acc = np.zeros((E.shape[0], U.shape[1]), dtype=np.float32)
        for a, b in ((2, 0), (1, 1), (0, 2), (1, 0), (0, 1), (0, 0)):   # smallest products first
            acc += ep[a] @ up[b]
        return acc.astype(np.float64)
    npieces, kc = {"bf16x4c32": (4, 32), "bf16x4c16": (4, 16), "bf16x3c32": (3, 32)}[rung]
    ep, up = _pieces(E, npieces), _pieces(U, npieces)
    m, K = E.shape
    pad = (-K) % kc
    acc = np.zeros((m, U.shape[1]))
    for a in range(npieces):
        for b in range(npieces - a):
            ea = np.pad(ep[a], ((0, 0), (0, pad))).reshape(m, -1, kc)
            ub = np.pad(up[b], ((0, pad), (0, 0))).reshape(-1, kc, U.shape[1])
            part = np.einsum("mck,ckb->cmb", ea, ub, optimize=True)     # float32 sums inside a chunk
            acc += part.astype(np.float64).sum(axis=0)                   # float64 across chunks
    return acc


def blocked_solve(W, U, bits, group, block, rung):
    """The GPU's scheme: per block the lazy update (in the rung's arithmetic), then the float64 column walk."""
    m, n = W.shape
    maxq = float(2 ** bits - 1)
    E = np.zeros((m, n))
    codes = np.zeros((m, n), np.uint8)
    scales = np.zeros((m, n // group), np.float32)
    zeros = np.zeros((m, n // group), np.uint8)
    pre = np.zeros((m, n))
    block = max(block, group)
    for i1 in range(0, n, block):
        i2 = min(n, i1 + block)
        S = W[:, i1:i2] - lazy_update(E[:, :i1], U[:i1, i1:i2], rung)
        for j in range(i1, i2):
            c = j - i1
            if j % group == 0:
                scale, zero, _, _, _ = orc.group_grid(S[:, c:c + group], int(maxq))
                scales[:, j // group] = scale.astype(np.float32)
                zeros[:, j // group] = zero.astype(np.uint8)
            w = S[:, c]
            x = w / scale
            pre[:, j] = x
            cd = np.clip(np.rint(x) + zero, 0.0, maxq)
            e = (w - scale * (cd - zero)) / U[j, j]
            if c + 1 < i2 - i1:
                S[:, c + 1:] -= np.outer(e, U[j, j + 1:i2])
            codes[:, j] = cd.astype(np.uint8)
            E[:, j] = e
    return codes, scales, zeros, pre


def ladder(W64, U, bits, group, block, rungs):
    base = orc.quantize_layer(W64, U, bits, group, want_pre=True)
    rows = []
    for rung in rungs:
        codes, scales, zeros, pre = blocked_solve(W64, U, bits, group, block, rung)
        rep = compare_quantization(W64, U, bits, group, None, codes, scales, zeros)
        same = np.all(codes == base["codes"], axis=1)
        dev = np.abs(pre[same] - base["pre_x"][same])
        rows.append(dict(rung=rung, exact_rows=int(rep["exact_rows"]),
                         flagged=int(rep["flagged_codes"] + rep["flagged_zeros"] + rep["flagged_scales"]),
                         unflagged=int(rep["unflagged"]), dev_rms=float(np.sqrt(np.mean(dev ** 2))) if dev.size else None))
    return rows


def test_only_float64_updates_reproduce_the_oracle_on_configuration_one():
    cfg = wl.CONFIGS["C1"]
    spec = cfg.layers[0]
    W64 = wl.to_f64(wl.gen_weight(spec))
    Hd, _ = orc.damp(orc.hessian(wl.to_f64(wl.gen_activations(spec))), cfg.damps[0])
    U = orc.inverse_cholesky_upper(Hd)
    rows = ladder(W64, U, cfg.bits, cfg.group, cfg.block, ["f64", "bf16x4c16", "bf16x4c32", "f32", "bf16"])
    for r in rows:
        print(r)
    by = {r["rung"]: r for r in rows}
    assert by["f64"]["exact_rows"] == spec.m and by["f64"]["flagged"] == 0 and by["f64"]["unflagged"] == 0
    for rung in ("bf16x4c16", "bf16x4c32", "f32"):
        assert by[rung]["flagged"] + by[rung]["unflagged"] >= 10 and 1e-9 < by[rung]["dev_rms"] < 1e-5
    assert by["f32"]["unflagged"] > 0
    assert by["bf16"]["unflagged"] == spec.m      # one bfloat16 piece: every row fails outright


if __name__ == "__main__":      # the full-size table: python tests/test_update_precision_ladder.py C2|C4|C3d
    import sys
    which = sys.argv[1]
    cfgname, layer, t_test, nrows = {"C2": ("C2", 0, 8192, 256), "C4": ("C4", 0, 8192, 256), "C3d": ("C3", 1, 12288, 128)}[which]
    cfg = wl.CONFIGS[cfgname]
    spec = cfg.layers[layer]
    sub = wl.scaled(spec, t=t_test)
    W64 = wl.to_f64(wl.gen_weight(sub))
    H = orc.hessian(wl.to_f64(wl.gen_activations(sub)))
    pick = np.sort(np.random.default_rng(5).choice(spec.m, nrows, replace=False))
    for damp in cfg.damps:
        U = orc.inverse_cholesky_upper(orc.damp(H, damp)[0])
        for r in ladder(W64[pick], U, cfg.bits, cfg.group, cfg.block,
                        ["f64", "bf16x4c16", "bf16x4c32", "f32", "bf16x3", "bf16"]):
            print(which, "damp", damp, r, flush=True)
