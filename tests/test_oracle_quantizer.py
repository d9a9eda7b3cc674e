"""Pins for the oracle's round-to-nearest min-max group quantizer (no GPU).

The paper names the scheme (min-max, round-to-nearest, group-wise with a scale and a
zero-point per group: Sec. 3.1, Sec. 6.1, App. C) and prints no worked example, so the
pins are known-answer grids, the textbook error bound and hand-computed small cases.
"""
import numpy as np
import pytest

from oracle import qeft_oracle as qo


def _deq(codes, scales, zeros, g):
    weak = np.zeros((codes.shape[0], 0), dtype=np.float16)
    return qo.dequantize(codes, scales, zeros, weak, g)


@pytest.mark.parametrize("bits", [3, 4])
def test_known_answer_grid_is_recovered(bits):
    """Weights that already lie on a grid s*(q-z) with a power-of-two s, whose group holds
    both end codes, must come back as exactly (q, s, z)."""
    r = np.random.default_rng(7)
    qmax = (1 << bits) - 1
    oc, g, ng = 6, 16, 3
    q = r.integers(0, qmax + 1, size=(oc, g * ng)).astype(np.int64)
    z = r.integers(0, qmax + 1, size=(oc, ng)).astype(np.int64)
    s = 2.0 ** r.integers(-9, -3, size=(oc, ng))
    for gi in range(ng):                      # plant both ends of the range in every group
        q[:, gi * g] = 0
        q[:, gi * g + 1] = qmax
    w = (s.repeat(g, axis=1) * (q - z.repeat(g, axis=1))).astype(np.float16)
    codes, scales, zeros, weak = qo.quantize_rtn(w, 0, bits, g)
    assert np.array_equal(codes, q.astype(np.uint8))
    assert np.array_equal(scales.astype(np.float64), s)
    assert np.array_equal(zeros.astype(np.float64), z.astype(np.float64))
    assert weak.shape == (oc, 0)


def test_hand_computed_group():
    """One group of four weights, 4-bit, worked on paper with exact fractions:
    fp16(-0.3) = -0.300048828125, fp16(0.45) = 0.449951171875, so hi - lo = 0.75 exactly and
    (hi-lo)/15 = 0.05 -> nearest fp16 is 1638 * 2^-15 = 0.04998779296875 (0.05 / 2^-15 = 1638.4).
    z = rint(0.300048828125 / s = 6.0024) = 6
    w/s = [-6.0024, 2.0, 9.0012, 0] -> q = [-6, 2, 9, 0] + 6 = [0, 8, 15, 6]."""
    w = np.array([[-0.3, 0.1, 0.45, 0.0]], dtype=np.float16)
    codes, scales, zeros, _ = qo.quantize_rtn(w, 0, 4, 4)
    assert codes.tolist() == [[0, 8, 15, 6]]
    assert float(zeros[0, 0]) == 6.0
    assert float(scales[0, 0]) == 1638 * 2.0 ** -15


def test_round_half_to_even_and_clipping():
    # s = 1 exactly (range 0..15): 2.5 -> 2, 3.5 -> 4 ; all-positive group has z = 0
    w = np.array([[0.0, 15.0, 2.5, 3.5, 0.5, 1.5]], dtype=np.float16)
    codes, scales, zeros, _ = qo.quantize_rtn(w, 0, 4, 8)
    assert float(scales[0, 0]) == 1.0 and float(zeros[0, 0]) == 0.0
    assert codes.tolist() == [[0, 15, 2, 4, 0, 2]]
    # all-negative group: lo = -15, hi = 0 -> z = 15
    codes, scales, zeros, _ = qo.quantize_rtn((-w).astype(np.float16), 0, 4, 8)
    assert float(zeros[0, 0]) == 15.0
    assert codes.tolist() == [[15, 0, 13, 11, 15, 13]]   # rint(-2.5)=-2, rint(-3.5)=-4, rint(-0.5)=-0, rint(-1.5)=-2


def test_all_zero_group_and_partial_last_group():
    w = np.zeros((2, 11), dtype=np.float16)
    w[1, 8:] = [0.5, -0.25, 0.125]            # the partial group (3 wide) of row 1
    codes, scales, zeros, weak = qo.quantize_rtn(w, 1, 4, 8)   # Kq = 10: groups [0,8) and [8,10)
    assert codes.shape == (2, 10) and scales.shape == (2, 2) and weak.shape == (2, 1)
    assert np.all(codes[0] == 0) and np.all(scales[0] == 1) and np.all(zeros[0] == 0)
    # row 1, partial group: statistics over the two real members only (0.5, -0.25); the
    # third value (0.125) is the weak column and is copied untouched
    assert float(weak[1, 0]) == 0.125
    assert float(scales[1, 1]) == 1638 * 2.0 ** -15      # fp16(0.75 / 15), as in the case above
    assert float(zeros[1, 1]) == 5.0
    assert codes[1, 8:].tolist() == [15, 0]


@pytest.mark.parametrize("bits", [3, 4])
def test_error_bound_and_ranges(bits):
    """|w - s*(q-z)| <= s/2 * (1 + qmax*2^-10): half a step, plus the fp16 rounding of s
    accumulated over at most qmax steps.  Zero is represented exactly."""
    r = np.random.default_rng(11)
    oc, ic, k, g = 24, 300, 12, 128
    w = (r.standard_normal((oc, ic)) * 0.02).astype(np.float16)
    codes, scales, zeros, weak = qo.quantize_rtn(w, k, bits, g)
    qmax = (1 << bits) - 1
    assert codes.max() <= qmax and zeros.max() <= qmax and zeros.min() >= 0
    assert np.array_equal(zeros, np.rint(zeros))
    assert np.array_equal(weak, w[:, ic - k:])
    wd = qo.dequantize(codes, scales, zeros, weak, g)
    s_full = scales.astype(np.float64).repeat(g, axis=1)[:, :ic - k]
    err = np.abs(wd[:, :ic - k] - w[:, :ic - k].astype(np.float64))
    assert np.all(err <= s_full * (0.5 + qmax * 2.0 ** -10))
    assert np.array_equal(wd[:, ic - k:], w[:, ic - k:].astype(np.float64))
    # the code equal to the zero-point dequantizes to exactly 0
    zc = zeros.astype(np.uint8).repeat(g, axis=1)[:, :ic - k]
    assert np.all(_deq(zc, scales, zeros, g) == 0)
    # each group uses its full range: both end codes appear (min-max scaling)
    for gi in range(scales.shape[1]):
        blk = codes[:, gi * g:(gi + 1) * g]
        assert np.all(blk.min(axis=1) == 0) and np.all(blk.max(axis=1) >= qmax - 1)


def test_quantizing_twice_is_stable():
    """Re-quantizing the dequantized weight reproduces the same stored form whenever the
    dequantized values are exact in fp16 (power-of-two scales)."""
    r = np.random.default_rng(5)
    w = (r.integers(-7, 9, size=(5, 64)) * 2.0 ** -6).astype(np.float16)
    w[:, 0] = -7 * 2.0 ** -6
    w[:, 1] = 8 * 2.0 ** -6
    c1, s1, z1, k1 = qo.quantize_rtn(w, 0, 4, 64)
    w2 = qo.dequantize(c1, s1, z1, k1, 64).astype(np.float16)
    assert np.array_equal(w2, w)
    c2, s2, z2, _ = qo.quantize_rtn(w2, 0, 4, 64)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2) and np.array_equal(z1, z2)


def test_codes_for_given_parameters_hand_cases():
    """Codes under parameters that did not come from min-max: s = 0.5, z = 3 on a hand-made row
    (w / s = [-7, -2.5, 0.5, 1.5, 30] -> rint half-to-even [-7, -2, 0, 2, 30] -> + 3, clipped to 0..15),
    and a second group with s = 0.25, z = 0."""
    w = np.array([[-3.5, -1.25, 0.25, 0.75, 15.0, 0.5, 0.125, 3.9, -1.0, 0.0, 7.0]], dtype=np.float16)
    s = np.array([[0.5, 0.25]], dtype=np.float16)
    z = np.array([[3.0, 0.0]], dtype=np.float16)
    codes = qo.codes_for_params(w, 1, 4, 5, s, z)        # Kq = 10: groups [0, 5) and [5, 10); column 10 is weak
    assert codes.tolist() == [[0, 1, 3, 5, 15, 2, 0, 15, 0, 0]]   # 0.125/0.25 = 0.5 -> 0; 3.9/0.25 = 15.6 -> 15 (clipped from 16)
    # the min-max quantizer's own codes are the codes under its own parameters
    r = np.random.default_rng(2)
    w = (r.standard_normal((9, 70)) * 0.02).astype(np.float16)
    c, sc, zp, _ = qo.quantize_rtn(w, 6, 3, 32)
    assert np.array_equal(qo.codes_for_params(w, 6, 3, 32, sc, zp), c)
