"""Pins for oracle/artifact_oracle.py: Eq. 12 against the numbers the paper prints, the bit
packing against hand-worked words, the inference form against the dense definition."""
import numpy as np
import pytest

from oracle import artifact_oracle as ao
from oracle import lopro_oracle as lo
from oracle import r1svd_oracle as ro

LLAMA2_7B = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
LLAMA2_13B = [(5120, 5120)] * 4 + [(13824, 5120)] * 2 + [(5120, 13824)]


def _printed_bit_widths():
    """tests/golden/average_bits.txt: the values the paper prints, with where it prints them."""
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "average_bits.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                model, bits, what, value = line.split()
                rows.append((model, int(bits), what, float(value)))
    return rows


def test_eq12_reproduces_the_papers_bit_widths():
    shapes = {"llama2-7b": LLAMA2_7B, "llama2-13b": LLAMA2_13B}
    rows = _printed_bit_widths()
    assert len(rows) == 4
    for model, bits, what, want in rows:
        # rank 16, fp8 factors, group 128, 16-bit scales; "terms=4" is Eq. 12 without the two terms the
        # paper calls negligible, "terms=2" without the low-rank terms as well
        full = ao.model_average_bits(shapes[model], bits, 16, 128, 16, 8, terms=4)
        if what == "low_rank":
            assert round(full - ao.model_average_bits(shapes[model], bits, 16, 128, 16, 8, terms=2), 2) == want
        else:
            assert round(full, 2) == want
    # and those two terms are indeed small: under a hundredth of a bit
    assert ao.model_average_bits(LLAMA2_7B, 2, 16, 128, 16, 8) - ao.model_average_bits(
        LLAMA2_7B, 2, 16, 128, 16, 8, terms=4) < 0.01


def test_eq12_term_by_term_on_a_square_layer():
    # m = n = 4096, 2 bits, group 128, 16-bit originals, rank 16 in 8 bits
    got = ao.average_bits(4096, 4096, 2, 16, 128, 16, 8)
    want = 2 + 16 / 128 + 2 * (16 * 8 / 4096) + 2 * 16 / 4096 + 16 * 16 / 4096 ** 2
    assert got == pytest.approx(want, rel=1e-15)
    # rank 0 and no groups: just the codes plus the two vectors
    assert ao.average_bits(512, 1024, 4, 16, 1024, 0, 8) == pytest.approx(4 + 16 / 1024 + 32 / 1024)


def test_packing_hand_worked_words():
    # 2 bits: codes 1,2,3,0 -> 0b00_11_10_01 = 0x39 in the low byte of the chunk's first word
    c = np.zeros((1, 32), dtype=np.uint8)
    c[0, :4] = [1, 2, 3, 0]
    p = ao.pack_codes(c, 2)
    assert p.shape == (1, 1, 2) and p[0, 0, 0] == 0x39 and p[0, 0, 1] == 0
    c[0, 16] = 2                                   # the 17th code opens the second word
    assert ao.pack_codes(c, 2)[0, 0, 1] == 2
    # 4 bits: codes 0xA, 0xB, 0xC -> 0xCBA
    c = np.zeros((1, 32), dtype=np.uint8)
    c[0, :3] = [0xA, 0xB, 0xC]
    assert ao.pack_codes(c, 4)[0, 0, 0] == 0xCBA
    # 3 bits: code 10 occupies bits 30..32 and straddles the first two words
    c = np.zeros((1, 32), dtype=np.uint8)
    c[0, 10] = 0b101
    p = ao.pack_codes(c, 3)
    assert p.shape == (1, 1, 3) and p[0, 0, 0] == (0b01 << 30) and p[0, 0, 1] == 0b1 and p[0, 0, 2] == 0
    c[0, 31] = 0b111
    assert ao.pack_codes(c, 3)[0, 0, 2] == (0b111 << 29)
    # chunk-major: the second chunk of every row comes after the first chunk of all rows
    c = np.zeros((3, 64), dtype=np.uint8)
    c[2, 32] = 3
    p = ao.pack_codes(c, 2)
    assert p.shape == (2, 3, 2) and p[1, 2, 0] == 3 and p.sum() == 3


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_packing_round_trip_and_size(bits):
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 2 ** bits, size=(7, 160), dtype=np.uint8)
    p = ao.pack_codes(codes, bits)
    assert p.dtype == np.uint32 and p.shape == (5, 7, bits) and p.size * 32 == codes.size * bits
    assert np.array_equal(ao.unpack_codes(p, bits, 160), codes)


def test_inference_form_equals_the_dense_layer():
    # Eq. 7: X W_hat^T with W_hat = W_r + Q(R') Q^T P^T, against the form that rotates X instead
    rng = np.random.default_rng(41)
    m, n, b, r, bits, group, bI, bH = 24, 128, 5, 3, 3, 32, 32, 32
    codes = rng.integers(0, 8, size=(m, n), dtype=np.uint8)
    scales = rng.uniform(0.01, 0.1, size=(m, n // group)).astype(np.float32)
    zeros = rng.integers(0, 8, size=(m, n // group), dtype=np.uint8)
    perm = rng.permutation(n)
    Uc = ro.e4m3_encode(ro.e4m3_round(rng.uniform(-0.4, 0.4, (r, m)))[0])
    Vc = ro.e4m3_encode(ro.e4m3_round(rng.uniform(-0.4, 0.4, (r, n)))[0])
    sigma = np.array([12.0, 5.5, 2.25])
    s = rng.uniform(0.3, 3.0, n)
    X = rng.standard_normal((b, n))
    Rq_rot = ao.dequantize(codes, scales, zeros, group)
    W_hat = ro.low_rank_weight({"U": ro.e4m3_decode(Uc), "V": ro.e4m3_decode(Vc), "sigma": sigma}, s) \
        + lo.unrotate_weight(Rq_rot, perm, bI, bH)
    got = ao.linear_forward(X, ao.pack_codes(codes, bits), bits, scales, zeros, group, perm, bI, bH, Uc, Vc, sigma, s)
    assert np.allclose(got, X @ W_hat.T, rtol=1e-12, atol=1e-12)
    # the pieces: no low-rank part, identity order and no rotation reduce to a plain dequantized product
    plain = ao.linear_forward(X, ao.pack_codes(codes, bits), bits, scales, zeros, group, np.arange(n), n, bH,
                              Uc[:0], Vc[:0], sigma[:0], s)
    assert np.allclose(plain, X @ Rq_rot.T, rtol=1e-13, atol=1e-13)


def test_stored_bits_counts_what_is_kept():
    # 4096 x 4096, 2 bits, group 128, rank 16: codes 2, scale+zero 40/128, factors 2*16*8/4096, vectors 96/4096
    got = ao.stored_bits(4096, 4096, 2, 128, 16)
    assert got == pytest.approx(2 + 40 / 128 + 2 * 16 * 8 / 4096 + 16 * 16 / 4096 ** 2 + 96 / 4096, rel=1e-12)
