"""Pins for the dense 3-bit layout of the oracle (32 codes in 3 words; what the 3-bit model
sizes of Tab. 5 imply).  Checked against things other than the oracle's own routines:
hand-written words, Python big-integer arithmetic, closed-form sizes, and the canonical
layout's unpack for the same codes."""
import numpy as np
import pytest

from oracle import qeft_oracle as qo


def test_hand_written_words():
    # codes 1, 2, ..., 7, 0, 1, ... : bit string built by hand.
    # codes 0..10 = 1,2,3,4,5,6,7,0,1,2,3 -> word 0 holds codes 0..9 in bits 0..29 and the low two bits of code 10
    codes = np.array([[(j + 1) % 8 for j in range(12)]], dtype=np.uint8)
    w = qo.pack_codes_dense3(codes, 16)
    w0 = 0
    for j in range(10):
        w0 |= ((j + 1) % 8) << (3 * j)
    w0 |= (3 & 0x3) << 30                     # code 10 = 3 = 0b011: bits 30, 31 hold its two low bits
    w1 = (3 >> 2) | (4 << 1)                  # its high bit, then code 11 = 4 at bits 1..3 of word 1
    assert int(w[0, 0]) == w0 and int(w[0, 1]) == w1
    assert not w[0, 2:].any()


def test_octet_is_three_bytes():
    # eight codes fill exactly three bytes: c0 | c1<<3 | ... | c7<<21
    codes = np.array([[7, 0, 5, 2, 1, 6, 3, 4]], dtype=np.uint8)
    w = qo.pack_codes_dense3(codes, 16)
    assert int(w[0, 0]) == sum(int(c) << (3 * i) for i, c in enumerate(codes[0]))
    assert int(w[0, 0]) < (1 << 24)


@pytest.mark.parametrize("kq", [1, 7, 10, 11, 31, 32, 33, 64, 120, 129, 1000])
def test_against_big_integers(kq):
    r = np.random.default_rng(kq)
    codes = r.integers(0, 8, (5, kq), dtype=np.uint8)
    lay = qo.layout(5, kq, 0, 3, 128, dense=True)
    assert lay["words_per_row"] == (3 * kq + 31) // 32
    w = qo.pack_codes_dense3(codes, lay["row_stride_words"])
    for o in range(5):
        n = sum(int(c) << (3 * j) for j, c in enumerate(codes[o]))
        ref = np.frombuffer(n.to_bytes(4 * lay["row_stride_words"], "little"), dtype="<u4")
        assert np.array_equal(w[o], ref)
        # and back, one code at a time, from the integer
        back = [(n >> (3 * j)) & 7 for j in range(kq)]
        assert back == qo.unpack_codes_dense3(w, kq)[o].tolist()


def test_three_bits_per_weight():
    # Llama-2 7B linear layers at 3.0 bits: 6 476 005 376 weights -> 2 428 502 016 bytes of codes (Tab. 5's
    # 3-bit sizes; ten codes per word need 6.7 % more).  Counted in used words: rows are then padded to 64 bytes.
    shapes = [(4096, 4096)] * 4 + [(11008, 4096)] * 2 + [(4096, 11008)]
    dense = sum(oc * qo.layout(oc, ic, 0, 3, 128, dense=True)["words_per_row"] * 4 for oc, ic in shapes) * 32
    canon = sum(oc * qo.layout(oc, ic, 0, 3, 128)["words_per_row"] * 4 for oc, ic in shapes) * 32
    assert dense == 2_428_502_016 == 6_476_005_376 * 3 // 8
    assert canon > 2_590_000_000
    lay = qo.layout(4096, 4096, 128, 3, 128, dense=True)
    assert lay["words_per_row"] == 372 and lay["row_stride_words"] == 384     # 3968 * 3 / 32, padded to 16 words
    assert lay["qweight_bytes"] == 4096 * 384 * 4
    with pytest.raises(ValueError):
        qo.layout(8, 64, 0, 4, 128, dense=True)


def test_same_codes_as_canonical_layout():
    r = np.random.default_rng(3)
    codes = r.integers(0, 8, (9, 517), dtype=np.uint8)
    a = qo.unpack_codes(qo.pack_codes(codes, 3, qo.layout(9, 517, 0, 3, 128)["row_stride_words"]), 517, 3)
    b = qo.unpack_codes_dense3(qo.pack_codes_dense3(codes, qo.layout(9, 517, 0, 3, 128, dense=True)["row_stride_words"]), 517)
    assert np.array_equal(a, codes) and np.array_equal(b, codes)


def test_samples_read_the_dense_layout():
    # sampled forward / input-gradient values through the dense layout equal the products with the dequantized matrix
    r = np.random.default_rng(5)
    oc, ic, k, g = 24, 300, 12, 128
    kq = ic - k
    lay = qo.layout(oc, ic, k, 3, g, dense=True)
    codes = r.integers(0, 8, (oc, kq), dtype=np.uint8)
    scales = (r.random((oc, lay["n_groups"])) * 0.01 + 0.001).astype(np.float16)
    zeros = r.integers(0, 8, (oc, lay["n_groups"])).astype(np.float16)
    weak = (r.standard_normal((oc, k)) * 0.02).astype(np.float16)
    qw = qo.pack_codes_dense3(codes, lay["row_stride_words"])
    w = qo.dequantize(codes, scales, zeros, weak, g)
    x = r.standard_normal((3, ic)).astype(np.float16)
    dy = r.standard_normal((3, oc)).astype(np.float16)
    pairs = [(0, 0), (2, oc - 1), (1, 7)]
    assert np.allclose(qo.fwd_samples(qw, scales, zeros, weak, kq, "3d", g, x, pairs),
                       [qo.linear_fwd(w, x)[m, o] for m, o in pairs], rtol=1e-12, atol=1e-12)
    pairs = [(0, 0), (1, 10), (2, 11), (0, 21), (1, kq - 1), (2, kq), (0, ic - 1)]   # columns 10, 21: codes that straddle words
    assert np.allclose(qo.bwd_dx_samples(qw, scales, zeros, weak, kq, "3d", g, dy, pairs),
                       [qo.linear_bwd_dx(w, dy)[m, c] for m, c in pairs], rtol=1e-12, atol=1e-12)
