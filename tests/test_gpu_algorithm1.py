"""Algorithm 1 of the paper for one layer, every stage on the GPU: activation scale, scaled rank-one
sketch (low-rank part + residual), column order, partial rotation of the residual and the Hessian,
damped factor, column solve, way back, layer error -- held against the oracles stage by stage with
the GPU's own upstream results, and against the identities that tie the stages together (Eq. 4, 7, 8)."""
import numpy as np
import pytest
import torch

import paper_2601_19675_amd as ptq
import ptq_workloads as wl
from oracle import lopro_oracle as lo
from oracle import ptq_oracle as orc
from oracle import r1svd_oracle as ro
from parity import compare_quantization, follow_r1svd, to_device

pytestmark = pytest.mark.gpu


def _t(shape, dtype):
    return torch.empty(shape, dtype=dtype, device="cuda")


@pytest.mark.parametrize("bits", [2, 3])
def test_one_layer_through_every_stage(bits, capsys):
    m, n, t, r, it, bI, bH, group, block = 96, 1024, 4096, 8, 4, 256, 256, 128, 128
    spec = wl.LayerSpec("alg1", m, n, t, dtype="bf16", x_sigma=1.0, layer_id=990)
    Ws = wl.gen_weight_with_low_rank_part(spec, rank=4)
    Xs = wl.gen_activations(spec)
    S = wl.gen_sketch_vectors(spec, r)
    W64, X64 = wl.to_f64(Ws), wl.to_f64(Xs)
    Wd, Xd = to_device(Ws), to_device(Xs)

    # ---- GPU chain --------------------------------------------------------------------------
    H = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    ptq.ptq_hessian_accumulate(H, Xd)
    asum = torch.zeros(n, dtype=torch.float64, device="cuda")
    ptq.ptq_activation_abs_sum(asum, Xd)
    s = _t(n, torch.float64)
    ptq.ptq_activation_scale(asum, t, s)
    U8, V8, sg, R = _t((r, m), torch.uint8), _t((r, n), torch.uint8), _t(r, torch.float16), _t((m, n), torch.float32)
    ptq.ptq_scaled_r1svd(Wd, s, to_device(S), it, U8, V8, sg, R)
    perm = _t(n, torch.int32)
    ptq.ptq_lopro_column_order(R, H, perm)
    Rr, Hr = _t((m, n), torch.float64), _t((n, n), torch.float64)
    ptq.ptq_lopro_rotate_weight(R, perm, bI, bH, Rr)
    ptq.ptq_lopro_rotate_hessian(H, perm, bI, bH, Hr)
    Uf, dead, info = _t((n, n), torch.float64), _t(n, torch.uint8), _t(2, torch.int32)
    ptq.ptq_damped_cholesky_inv(Hr, 0.01, Uf, dead, info)
    codes, scales = _t((m, n), torch.uint8), _t((m, n // group), torch.float32)
    zeros, Rq_rot = _t((m, n // group), torch.uint8), _t((m, n), torch.float64)
    ptq.ptq_quantize_layer(Rr, Uf, dead, bits, group, block, codes, scales, zeros, Rq_rot, None)
    Rq = _t((m, n), torch.float64)
    ptq.ptq_lopro_unrotate_weight(Rq_rot, perm, bI, bH, Rq)
    e_rot, e_res = torch.zeros(3, dtype=torch.float64, device="cuda"), torch.zeros(3, dtype=torch.float64, device="cuda")
    ptq.ptq_layer_error(Rr, Rq_rot, Hr, e_rot)      # loss of the rotated residual under H'
    ptq.ptq_layer_error(R, Rq, H, e_res)            # the same residual in the layer's own basis under H
    torch.cuda.synchronize()
    assert info.cpu().tolist() == [0, 0]

    # ---- identities between the stages ----------------------------------------------------------
    s_g, R_g = s.cpu().numpy(), R.cpu().numpy().astype(np.float64)
    out = {"U": ro.e4m3_decode(U8.cpu().numpy()), "V": ro.e4m3_decode(V8.cpu().numpy()),
           "sigma": sg.cpu().numpy().astype(np.float64)}
    W_r = ro.low_rank_weight(out, s_g)
    # Eq. 4: W = W_r + R for what is stored, up to the float32 roundings of the running matrix
    bound = (np.abs(W64 * s_g) + np.abs(out["U"]).T @ (np.abs(out["V"]) * out["sigma"][:, None])) / s_g
    assert np.all(np.abs(W_r + R_g - W64) <= (r + 3) * 2.0 ** -24 * bound)
    # Eq. 8: the residual's loss is the same number in both bases (tr(D H D^T) itself, entry 1 of the output)
    # (the rotated residual is float64 and takes the float64 form of the sum, the float32 residual the form with
    # two bfloat16 pieces per operand, whose traces hold to about 1e-6)
    assert float(e_rot[1]) == pytest.approx(float(e_res[1]), rel=4e-6)
    # Eq. 7: the layer that inference would run, W_r + Q(R') Q^T P^T, and its error against W under H,
    # evaluated by the oracle from the GPU's outputs: W - W_hat = R - Rq, so it is the residual's loss
    H_ref = orc.hessian(X64)
    W_hat = W_r + Rq.cpu().numpy()
    rel_layer, num, den = orc.layer_error(W64, W_hat, H_ref)
    assert num == pytest.approx(float(e_res[1]), rel=2e-4)     # float32 residual, float32-accumulated H

    # ---- each stage against its oracle, fed the GPU's upstream results ---------------------------
    assert np.allclose(s_g, ro.activation_scale(ro.mean_abs_activation(X64)), rtol=1e-12)
    ref = follow_r1svd(W64, s_g, S.astype(np.float64), it, U8.cpu().numpy(), V8.cpu().numpy(), out["sigma"], 2e-3)
    assert np.array_equal(ref["U_code"], U8.cpu().numpy()) and np.array_equal(ref["V_code"], V8.cpu().numpy())
    assert np.array_equal(ref["sigma"], out["sigma"]) and ref["followed"] <= 2
    Hg = orc.symmetrize_from_upper(H.cpu().numpy())
    pg = perm.cpu().numpy().astype(np.int64)
    keys_ref = lo.column_keys(Hg, R_g)
    pr = lo.permutation(keys_ref, True)
    assert sorted(pg.tolist()) == list(range(n))
    for c in np.nonzero(pg != pr)[0]:          # only keys that tie to rounding may swap places
        assert abs(keys_ref[pg[c]] - keys_ref[pr[c]]) <= 1e-12 * abs(keys_ref[pr[c]])
    assert np.array_equal(Rr.cpu().numpy(), lo.rotate_weight(R_g, pg, bI, bH))
    Hr_ref = lo.rotate_hessian(Hg, pg, bI, bH)
    dg = np.sqrt(np.diag(Hr_ref))
    assert np.max(np.abs(Hr.cpu().numpy() - Hr_ref) / np.outer(dg, dg)) <= 1e-13
    rep = compare_quantization(Rr.cpu().numpy(), Uf.cpu().numpy(), bits, group, None, codes.cpu().numpy(),
                               scales.cpu().numpy(), zeros.cpu().numpy())
    assert rep["unflagged"] == 0, rep["details"][:3]

    # ---- the stored layer applied to a few tokens (Eq. 7 as inference runs it) -------------------
    from oracle import artifact_oracle as ao
    packed = _t((n // 32, m, bits), torch.int32)
    st_, zt_ = _t((n // group, m), torch.float32), _t((n // group, m), torch.uint8)
    ptq.ptq_pack_codes(codes, bits, packed, scales, zeros, group, st_, zt_)
    tok = 6
    O = _t((tok, m), torch.float32)
    ptq.ptq_lopro_linear_forward(Xd[:tok], packed, bits, st_, zt_, group, perm, bI, bH, U8, V8, sg, s, O)
    torch.cuda.synchronize()
    O_g = O.cpu().numpy().astype(np.float64)
    O_hat = X64[:tok] @ W_hat.T                     # the dense layer built from the same stored parts
    O_true = X64[:tok] @ W64.T
    sc_ = np.repeat(scales.cpu().numpy().astype(np.float64), group, axis=1)
    cz_ = codes.cpu().numpy().astype(np.float64) + np.repeat(zeros.cpu().numpy().astype(np.float64), group, axis=1)
    mag = np.abs(lo.rotate_weight(X64[:tok], pg, bI, bH)) @ (sc_ * cz_).T \
        + (np.abs(X64[:tok] / s_g) @ np.abs(out["V"]).T * out["sigma"]) @ np.abs(out["U"])
    assert np.all(np.abs(O_g - O_hat) <= (120 + n // 256) * 2.0 ** -24 * mag + 1e-30)
    # and it approximates the original layer about as well as the layer error says
    rel_out = np.linalg.norm(O_g - O_true) / np.linalg.norm(O_true)
    assert rel_out < 3 * rel_layer
    assert ptq.ptq_average_bits(m, n, bits, 16, group, r, 8) == pytest.approx(
        ao.average_bits(m, n, bits, 16, group, r, 8), rel=1e-15)

    # ---- context (printed, not asserted: the paper's claim is about trained weights) -------------
    Hd_, dm = orc.damp(H_ref, 0.01)
    plain = orc.quantize_layer(W64, orc.inverse_cholesky_upper(Hd_), bits, group, dead=dm)
    rel_plain = orc.layer_error(W64, plain["Wq"], H_ref)[0]
    with capsys.disabled():
        print(f"  [{bits}-bit, {m}x{n}: relative layer error with low-rank part + rotation {rel_layer:.4f}, "
              f"plain column solve on W {rel_plain:.4f}]", flush=True)
    assert rel_layer < 1.0
