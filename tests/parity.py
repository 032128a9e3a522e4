"""Helpers shared by the GPU parity tests: tensor marshalling and the
near-tie protocol that compares GPU codes / scales / zeros with the oracle.

The column recurrence is chaotic per row: one code that rounds the other way
changes every later code of that row.  The acceptance rule is therefore
applied decision by decision, in the order the algorithm takes them (for each
group: scale, zero-point, then the group's codes).  At the first decision
where GPU and oracle differ, the oracle's pre-rounding value must lie within
`tol` of the rounding boundary and the GPU must have taken the neighbouring
value; that decision is then forced in the oracle, the row is solved again,
and the comparison continues.  Anything else is an unflagged mismatch.
"""
from __future__ import annotations

import numpy as np

from oracle import ptq_oracle as orc
from ptq_workloads import to_device, to_f64  # noqa: F401  (to_device is re-exported for the tests)


def hessian_errors(H_gpu: np.ndarray, H_ref: np.ndarray):
    """(Frobenius-relative error, max entry error scaled by sqrt(H_ii H_jj)) on the upper triangle."""
    iu = np.triu_indices_from(H_ref)
    d = H_gpu[iu] - H_ref[iu]
    fro = np.linalg.norm(d) / np.linalg.norm(H_ref[iu])
    dg = np.sqrt(np.abs(np.diag(H_ref)))
    sc = np.outer(dg, dg)[iu]
    sc[sc == 0] = 1.0
    return float(fro), float(np.max(np.abs(d) / sc))


def _first_mismatch(o, g_codes, g_scales, g_zeros, group):
    """Earliest differing decision of one row, in algorithm order, or None."""
    best = None
    ks = np.nonzero(o["scales"][0] != g_scales)[0]
    if ks.size:
        best = (int(ks[0]) * (group + 2), "scale", int(ks[0]))
    kz = np.nonzero(o["zeros"][0] != g_zeros)[0]
    if kz.size:
        c = (int(kz[0]) * (group + 2) + 1, "zero", int(kz[0]))
        best = c if best is None or c < best else best
    jc = np.nonzero(o["codes"][0] != g_codes)[0]
    if jc.size:
        j = int(jc[0])
        c = ((j // group) * (group + 2) + 2 + j % group, "code", j)
        best = c if best is None or c < best else best
    return best


def _alt_round(x):
    """The integer on the other side of the rounding boundary, and the distance to it."""
    f = np.floor(x)
    margin = abs((x - f) - 0.5)
    alt = f if np.rint(x) != f else f + 1.0
    return alt, margin


def oracle_solve_rows(W64, U, bits, group, dead=None, static_groups=False, chunk=128, workers=None):
    """orc.quantize_layer(..., want_pre=True) over all rows of W64, called on slices of `chunk` rows
    from a pool of threads: rows are independent given U, so the slices are separate oracle runs
    whose results are stacked.  (Nothing of the oracle is changed; a slice of 128 rows keeps the
    column loop's rank-one updates in cache, and numpy releases the interpreter lock inside them.)"""
    import os
    from concurrent.futures import ThreadPoolExecutor
    m = W64.shape[0]
    if m <= chunk:
        return orc.quantize_layer(W64, U, bits, group, dead=dead, want_pre=True, static_groups=static_groups)
    workers = workers or min(16, os.cpu_count() or 1)
    los = list(range(0, m, chunk))
    with ThreadPoolExecutor(workers) as ex:
        parts = list(ex.map(lambda lo: orc.quantize_layer(W64[lo:lo + chunk], U, bits, group, dead=dead, want_pre=True,
                                                          static_groups=static_groups), los))
    return {k: np.concatenate([p[k] for p in parts], axis=0) for k in parts[0]}


def compare_quantization(W64, U, bits, group, dead, g_codes, g_scales, g_zeros, tol=1e-5,
                         max_forced_per_row=64, static_groups=False):
    """Runs the protocol over all rows of W64.  Returns a report dict."""
    maxq = float(2 ** bits - 1)
    m, n = W64.shape
    base = oracle_solve_rows(W64, U, bits, group, dead, static_groups)
    rep = dict(rows=m, exact_rows=0, flagged_codes=0, flagged_zeros=0, flagged_scales=0,
               unflagged=0, max_scale_margin_ulp=0.0, details=[], oracle=base)
    for r in range(m):
        same = (np.array_equal(base["codes"][r], g_codes[r]) and
                np.array_equal(base["scales"][r], g_scales[r]) and
                np.array_equal(base["zeros"][r], g_zeros[r]))
        if same:
            rep["exact_rows"] += 1
            continue
        cur = {k: v[r:r + 1] for k, v in base.items()}
        forced = {}
        for _ in range(max_forced_per_row):
            mm = _first_mismatch(cur, g_codes[r], g_scales[r], g_zeros[r], group)
            if mm is None:
                break
            _, kind, idx = mm
            ok = False
            if kind == "code":
                k = idx // group
                alt, margin = _alt_round(cur["pre_x"][0, idx])
                altc = min(max(alt + float(cur["zeros"][0, k]), 0.0), maxq)
                ok = margin <= tol and float(g_codes[r, idx]) == altc
                val = int(g_codes[r, idx])
                rep["flagged_codes"] += ok
            elif kind == "zero":
                alt, margin = _alt_round(cur["pre_zero"][0, idx])
                ok = margin <= tol and float(g_zeros[r, idx]) == alt
                val = int(g_zeros[r, idx])
                rep["flagged_zeros"] += ok
            else:
                ps = cur["pre_scale"][0, idx]
                so = np.float32(ps)
                sg = np.float32(g_scales[r, idx])
                adjacent = sg in (np.nextafter(so, np.float32(np.inf)), np.nextafter(so, np.float32(-np.inf)))
                mid = 0.5 * (float(so) + float(sg))
                ulp = abs(float(sg) - float(so))
                margin = abs(ps - mid) / ulp if ulp > 0 else np.inf
                # the scale's pre-rounding value within relative tol of the float32 midpoint
                ok = bool(adjacent) and abs(ps - mid) <= tol * abs(ps)
                val = float(sg)
                if ok:
                    rep["flagged_scales"] += 1
                    rep["max_scale_margin_ulp"] = max(rep["max_scale_margin_ulp"], float(margin))
            if not ok:
                rep["unflagged"] += 1
                rep["details"].append((r, kind, idx))
                break
            forced[(kind, 0, idx)] = val
            cur = orc.quantize_layer(W64[r:r + 1], U, bits, group, dead=dead, forced=forced, want_pre=True,
                                     static_groups=static_groups)
        else:
            rep["unflagged"] += 1
            rep["details"].append((r, "too many forced decisions", -1))
    return rep


def stored_to_f64(a):
    return to_f64(a)


# ----------------------------------------------------------------------------
# the same idea for the low-rank sketch: near-ties of the stored e4m3 / fp16 values
# ----------------------------------------------------------------------------
def follow_r1svd(W64, s, S, it, U_codes, V_codes, sigma, tol, max_followed=4):
    """Oracle run of the scaled rank-one sketch that takes another implementation's stored value
    where -- and only where -- that value is itself a legitimate rounding of the oracle's own
    unrounded one: within (1/2 + tol) quanta of it, tol standing for the arithmetic noise of the
    implementation under test.  One flipped code changes every later rank, so decisions are
    settled rank by rank: the oracle is run, the first rank with a difference is examined, its
    near-ties are forced (the oracle's U_force / V_force / sigma_force), and the oracle is run
    again; anything that is not a near-tie stays different for the caller to see.  Gives up after
    `max_followed` forced values.  Returns the oracle's result with "followed" = their number."""
    from oracle import r1svd_oracle as ro
    r, m, n = S.shape[0], W64.shape[0], W64.shape[1]
    Uf = np.full((r, m), -1, dtype=np.int16)
    Vf = np.full((r, n), -1, dtype=np.int16)
    sf = np.full(r, np.nan)
    followed = 0
    settled = 0                      # ranks below this one agree or are given up on
    while True:
        ref = ro.scaled_r1svd(W64, s, S, it, U_force=Uf, V_force=Vf, sigma_force=sf)
        ref["followed"] = followed
        k = settled
        while k < r and (np.array_equal(ref["U_code"][k], U_codes[k]) and np.array_equal(ref["V_code"][k], V_codes[k])
                         and ref["sigma"][k] == sigma[k]):
            k += 1
        if k == r or followed >= max_followed:
            return ref
        took = 0
        for own, theirs, exact, force in ((ref["U_code"][k], U_codes[k], ref["U_exact"][k], Uf[k]),
                                          (ref["V_code"][k], V_codes[k], ref["V_exact"][k], Vf[k])):
            near = np.abs(ro.e4m3_decode(theirs) - exact) <= (0.5 + tol) * ro.quantum(exact, "e4m3")
            take = (own != theirs) & near & ((theirs & 0x7F) != 0x7F) & (force < 0)
            force[take] = theirs[take]
            took += int(np.count_nonzero(take))
        th = float(sigma[k])
        if (th != ref["sigma"][k] and np.isfinite(th) and np.isnan(sf[k]) and
                abs(th - ref["sigma_exact"][k]) <= (0.5 + tol) * float(ro.quantum(ref["sigma_exact"][k], "fp16"))):
            sf[k] = th
            took += 1
        followed += took
        if took == 0:
            settled = k + 1          # a real difference in rank k: leave it, look no further in this rank
            if settled == r:
                return ref


# ----------------------------------------------------------------------------
# the vector-quantized solve: near-ties of the assignment
# ----------------------------------------------------------------------------
def compare_vq(W64, U, codebook, dead, g_indices, tol=1e-5, max_forced_per_row=16):
    """The protocol of compare_quantization for the vector quantizer.  A group's decision is the entry
    with the smallest loss; the boundary between two entries is where their losses are equal, and a
    point at distance delta (in units of the entries' separation, both measured through T^-1) from it
    has a loss difference of 2 delta |(c_a - c_b) T^-1|^2.  At the first group where the GPU's index
    differs from the oracle's, the difference is accepted when the oracle's own losses put the point
    within `tol` of that boundary; the GPU's index is then forced and the row solved again."""
    from oracle import vq_oracle as vqo
    C = np.asarray(codebook, dtype=np.float64)
    d = C.shape[1]
    m = W64.shape[0]
    base = vqo.quantize_layer_vq(W64, U, C, dead=dead, want_margins=True)
    rep = dict(rows=m, exact_rows=0, flagged=0, unflagged=0, details=[], oracle=base, max_margin=0.0)
    for r in range(m):
        if np.array_equal(base["indices"][r], g_indices[r]):
            rep["exact_rows"] += 1
            continue
        cur = {k: v[r:r + 1] for k, v in base.items()}
        forced = {}
        for _ in range(max_forced_per_row):
            diff = np.nonzero(cur["indices"][0] != g_indices[r])[0]
            if diff.size == 0:
                break
            g = int(diff[0])
            j = g * d
            T = U[j:j + d, j:j + d]
            losses = vqo.group_losses(cur["pre_w"][0, j:j + d], C, T)
            ko, kg = int(cur["indices"][0, g]), int(g_indices[r, g])
            sep = float(np.sum(vqo.group_errors(C[kg][None, :], C[ko], T) ** 2))
            margin = (losses[kg] - losses[ko]) / (2.0 * sep) if sep > 0 else 0.0
            if kg >= C.shape[0] or margin > tol or (sep == 0.0 and kg > ko):
                rep["unflagged"] += 1
                rep["details"].append((r, g, ko, kg, float(margin)))
                break
            rep["flagged"] += 1
            rep["max_margin"] = max(rep["max_margin"], float(margin))
            forced[(0, g)] = kg
            cur = vqo.quantize_layer_vq(W64[r:r + 1], U, C, dead=dead, forced=forced, want_margins=True)
        else:
            rep["unflagged"] += 1
            rep["details"].append((r, -1, -1, -1, 0.0))
    return rep
