"""Pins for the oracle's dequantize / forward / backward (no GPU).

The paper prints no numeric example of a layer output, so the oracle is pinned by
(1) exact rational brute force written independently with Python ints and Fractions,
(2) special cases that reduce to a library GEMM on other code (torch CPU),
(3) algebraic identities that a dropped term, wrong sign, wrong group index or a
    transposed operand would break.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import synth


def _frac(h) -> Fraction:
    return Fraction(float(h))          # a float16 is a dyadic rational: exact


def _brute_weight(qweight, scales, zeros, weak, oc, ic, k, bits, g):
    """W[o][c] as exact Fractions straight from the packed words (Python ints only)."""
    per = 8 if bits == 4 else 10
    kq = ic - k
    W = [[None] * ic for _ in range(oc)]
    for o in range(oc):
        for c in range(ic):
            if c < kq:
                word = int(qweight[o][c // per])
                code = (word >> (bits * (c % per))) & ((1 << bits) - 1)
                W[o][c] = _frac(scales[o][c // g]) * (code - _frac(zeros[o][c // g]))
            else:
                W[o][c] = _frac(weak[o][c - kq])
    return W


CASES = [  # oc, ic, k, bits, g, m
    (3, 20, 4, 4, 8, 2),
    (3, 20, 4, 3, 8, 2),
    (2, 13, 6, 4, 16, 3),     # Kq = 7 < g: one partial group
    (4, 37, 5, 3, 12, 2),     # groups straddle 10-code words
    (2, 9, 0, 4, 4, 1),       # no weak column
    (2, 6, 6, 4, 4, 2),       # every column weak
]


@pytest.mark.parametrize("oc,ic,k,bits,g,m", CASES)
def test_against_exact_rational_brute_force(oc, ic, k, bits, g, m):
    r = np.random.default_rng(oc * 1000 + ic)
    lay = qo.layout(oc, ic, k, bits, g)
    kq, ng = lay["kq"], lay["n_groups"]
    codes = r.integers(0, 1 << bits, size=(oc, kq), dtype=np.uint8)
    scales = r.uniform(0.01, 0.1, size=(oc, ng)).astype(np.float16)
    zeros = r.uniform(0, (1 << bits) - 1, size=(oc, ng)).astype(np.float16)   # non-integer on purpose
    weak = r.standard_normal((oc, k)).astype(np.float16)
    x = r.standard_normal((m, ic)).astype(np.float16)
    dy = r.standard_normal((m, oc)).astype(np.float16)
    qweight = qo.pack_codes(codes, bits, lay["row_stride_words"])

    W = _brute_weight(qweight, scales, zeros, weak, oc, ic, k, bits, g)
    w64 = qo.dequantize(qo.unpack_codes(qweight, kq, bits), scales, zeros, weak, g)
    for o in range(oc):
        for c in range(ic):
            assert Fraction(w64[o, c]) == W[o][c]          # s*(q-z) is exact in float64

    y = qo.linear_fwd(w64, x)
    dx = qo.linear_bwd_dx(w64, dy)
    dw = qo.weak_grad(dy, x[:, kq:])
    for mi in range(m):
        for o in range(oc):
            ref = sum(_frac(x[mi, c]) * W[o][c] for c in range(ic))
            assert abs(Fraction(y[mi, o]) - ref) <= abs(ref) * Fraction(1, 10**12) + Fraction(1, 10**14)
        for c in range(ic):
            ref = sum(_frac(dy[mi, o]) * W[o][c] for o in range(oc))
            assert abs(Fraction(dx[mi, c]) - ref) <= abs(ref) * Fraction(1, 10**12) + Fraction(1, 10**14)
    for o in range(oc):
        for c in range(k):
            ref = sum(_frac(dy[mi, o]) * _frac(x[mi, kq + c]) for mi in range(m))
            assert abs(Fraction(dw[o, c]) - ref) <= abs(ref) * Fraction(1, 10**12) + Fraction(1, 10**14)
    # the sampled accessors agree with the full products
    pairs = [(mi, o) for mi in range(m) for o in range(oc)]
    assert np.allclose(qo.fwd_samples(qweight, scales, zeros, weak, kq, bits, g, x, pairs),
                       y.reshape(-1), rtol=1e-13, atol=1e-15)
    pairs = [(mi, c) for mi in range(m) for c in range(ic)]
    assert np.allclose(qo.bwd_dx_samples(qweight, scales, zeros, weak, kq, bits, g, dy, pairs),
                       dx.reshape(-1), rtol=1e-13, atol=1e-15)
    pairs = [(o, c) for o in range(oc) for c in range(k)]
    assert np.allclose(qo.weak_grad_samples(dy, x[:, kq:], pairs), dw.reshape(-1), rtol=1e-13, atol=1e-15)


def _layer(oc, ic, k, bits, g, seed):
    lay = qo.layout(oc, ic, k, bits, g)
    codes, scales, zeros = synth.make_codes(oc, lay["kq"], lay["n_groups"], bits, seed)
    weak = synth.make_weight(oc, ic, seed)[:, ic - k:].copy()
    return lay, codes, scales, zeros, weak


def test_all_columns_weak_is_a_plain_gemm():
    """k = IC: nothing is quantized and the layer is an ordinary FP16 linear layer."""
    oc, ic, m = 48, 96, 9
    w = synth.make_weight(oc, ic, 1)
    x = synth.make_activations(m, ic, 0, 1)
    codes, scales, zeros, weak = qo.quantize_rtn(w, ic, 4, 128)
    assert codes.shape == (oc, 0)
    w64 = qo.dequantize(codes, scales, zeros, weak, 128)
    ref = torch.from_numpy(x).double() @ torch.from_numpy(w).double().T
    assert np.allclose(qo.linear_fwd(w64, x), ref.numpy(), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("bits", [3, 4])
def test_no_weak_column_is_pure_group_quantization(bits):
    """k = 0 with one (s, z) shared by the whole matrix: Y = s * (X.Q^T - z * rowsum(X)),
    an integer-matrix GEMM done by torch, not by the oracle's elementwise formula."""
    oc, ic, m, g = 40, 256, 5, 128
    lay, codes, _, _, _ = _layer(oc, ic, 0, bits, g, 3)
    s, z = np.float16(0.0123), np.float16(3.0)
    scales = np.full((oc, lay["n_groups"]), s, dtype=np.float16)
    zeros = np.full((oc, lay["n_groups"]), z, dtype=np.float16)
    weak = np.zeros((oc, 0), dtype=np.float16)
    x = synth.make_activations(m, ic, 0, 3)
    xt = torch.from_numpy(x).double()
    ref = float(s) * (xt @ torch.from_numpy(codes.astype(np.float64)).T - float(z) * xt.sum(dim=1, keepdim=True))
    y = qo.linear_fwd(qo.dequantize(codes, scales, zeros, weak, g), x)
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)


def test_per_group_scales_pick_the_right_group():
    """Make all groups but one have scale 0: the output must be that group's slice of X
    times that group's codes.  A wrong group index (off by one, j % g instead of j // g)
    fails here."""
    oc, ic, k, g, m = 16, 5 * 32 + 8, 8, 32, 4
    lay, codes, scales, zeros, weak = _layer(oc, ic, k, 4, g, 4)
    x = synth.make_activations(m, ic, k, 4)
    weak[:] = 0
    for keep in range(lay["n_groups"]):
        sc = np.zeros_like(scales)
        sc[:, keep] = scales[:, keep]
        y = qo.linear_fwd(qo.dequantize(codes, sc, zeros, weak, g), x)
        sl = slice(keep * g, min((keep + 1) * g, lay["kq"]))
        wg = sc[:, keep:keep + 1].astype(np.float64) * (codes[:, sl].astype(np.float64) - zeros[:, keep:keep + 1].astype(np.float64))
        ref = torch.from_numpy(x[:, sl]).double() @ torch.from_numpy(wg).T
        assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-13)


def test_zero_scales_leave_only_the_weak_path():
    """s = 0 everywhere: Y = X[:, weak] . W_weak^T and dX is zero outside the weak block."""
    oc, ic, k, g, m = 32, 200, 24, 64, 6
    lay, codes, scales, zeros, weak = _layer(oc, ic, k, 4, g, 5)
    x = synth.make_activations(m, ic, k, 5)
    dy = synth.make_grad_output(m, oc, 5)
    w64 = qo.dequantize(codes, np.zeros_like(scales), zeros, weak, g)
    ref = torch.from_numpy(x[:, ic - k:]).double() @ torch.from_numpy(weak).double().T
    assert np.allclose(qo.linear_fwd(w64, x), ref.numpy(), rtol=1e-13, atol=1e-15)
    dx = qo.linear_bwd_dx(w64, dy)
    assert np.all(dx[:, :ic - k] == 0)
    refdx = torch.from_numpy(dy).double() @ torch.from_numpy(weak).double()
    assert np.allclose(dx[:, ic - k:], refdx.numpy(), rtol=1e-13, atol=1e-15)


def test_forward_is_additive_over_the_two_paths():
    oc, ic, k, g, m = 24, 300, 44, 128, 3
    lay, codes, scales, zeros, weak = _layer(oc, ic, k, 3, g, 6)
    x = synth.make_activations(m, ic, k, 6)
    w64 = qo.dequantize(codes, scales, zeros, weak, g)
    xq, xw = x.copy(), x.copy()
    xq[:, ic - k:] = 0
    xw[:, :ic - k] = 0
    y = qo.linear_fwd(w64, x)
    assert np.allclose(y, qo.linear_fwd(w64, xq) + qo.linear_fwd(w64, xw), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("bits", [3, 4])
def test_adjoint_identities_pin_the_backward(bits):
    """<dY, fwd(X)> = <bwd_dx(dY), X>  and  <dY, Xw.D^T> = <weak_grad(dY, Xw), D>: the
    backward products are the transposes of the forward map, whatever W is."""
    oc, ic, k, g, m = 56, 333, 21, 128, 7
    lay, codes, scales, zeros, weak = _layer(oc, ic, k, bits, g, 8)
    x = synth.make_activations(m, ic, k, 8)
    dy = synth.make_grad_output(m, oc, 8)
    w64 = qo.dequantize(codes, scales, zeros, weak, g)
    lhs = np.sum(dy.astype(np.float64) * qo.linear_fwd(w64, x))
    rhs = np.sum(qo.linear_bwd_dx(w64, dy) * x.astype(np.float64))
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), 1.0)
    d = np.random.default_rng(9).standard_normal((oc, k))
    xw = x[:, ic - k:]
    lhs = np.sum(dy.astype(np.float64) * (xw.astype(np.float64) @ d.T))
    rhs = np.sum(qo.weak_grad(dy, xw) * d)
    assert abs(lhs - rhs) <= 1e-11 * max(abs(lhs), 1.0)
    # finite-difference view of Eq. 5: moving W_weak by eps*D changes <dY, Y> by eps*<dW, D>
    eps = 2.0 ** -10
    w_shift = w64.copy()
    w_shift[:, ic - k:] += eps * d
    delta = np.sum(dy.astype(np.float64) * (qo.linear_fwd(w_shift, x) - qo.linear_fwd(w64, x)))
    assert abs(delta - eps * rhs) <= 1e-9 * abs(eps * rhs) + 1e-15


def test_exact_integer_case():
    """Scales in {1, 0.5}, integer zero-points, small integer X and W_weak: every product
    and partial sum is an integer or half-integer, so the fp16 result is exact and equals
    an int64 computation."""
    r = np.random.default_rng(12)
    oc, ic, k, g, m = 8, 64 + 8, 8, 32, 4
    codes = r.integers(0, 16, size=(oc, 64), dtype=np.uint8)
    scales = r.choice([1.0, 0.5], size=(oc, 2)).astype(np.float16)
    zeros = r.integers(0, 16, size=(oc, 2)).astype(np.float16)
    weak = r.integers(-3, 4, size=(oc, k)).astype(np.float16)
    x = r.integers(-2, 3, size=(m, ic)).astype(np.float16)
    w2 = np.concatenate([(2 * scales.astype(np.float64)).astype(np.int64).repeat(g, axis=1)
                         * (codes.astype(np.int64) - zeros.astype(np.int64).repeat(g, axis=1)),
                         2 * weak.astype(np.int64)], axis=1)          # 2*W as integers
    ref2 = x.astype(np.int64) @ w2.T
    y = qo.linear_fwd(qo.dequantize(codes, scales, zeros, weak, g), x)
    assert np.array_equal(2 * y, ref2.astype(np.float64))
    assert np.array_equal(qo.round_fp16(y).astype(np.float64) * 2, ref2.astype(np.float64))


def test_round_fp16_is_nearest_even():
    # 2049 is halfway between fp16 neighbours 2048 and 2050 -> even mantissa (2048); 2051 -> 2052
    assert qo.round_fp16(np.array([2049.0, 2051.0, 1e-8, 65519.0])).tolist() == [2048.0, 2052.0, 0.0, 65504.0]
    # no double rounding through float32: 1 + 2^-11 + 2^-30 is above the halfway point
    assert float(qo.round_fp16(np.array([1 + 2.0 ** -11 + 2.0 ** -30]))[0]) == 1 + 2.0 ** -10


def test_fp16_rounded_weights_leave_the_bar_on_eight_term_sums():
    """Why input gradients over fewer than 64 output channels must not round the dequantized weights: on these two
    seeded layers (8 output channels) the exact product with weights rounded once to fp16 - the best a kernel that
    feeds fp16 operands can do - puts an output outside the per-element bar 2e-3 (|r| + rms), while the same product
    with unrounded weights stays five times inside it.  The Frobenius error is 3e-4 either way."""
    from paper_2410_08661_amd import synth

    def worst(a, r):
        rms = float(np.sqrt(np.mean(r * r)))
        return float(np.max(np.abs(a - r) / (2e-3 * (np.abs(r) + rms))))

    for oc, ic, k, m, seed in [(8, 320, 256, 130, 14), (8, 640, 256, 260, 14)]:
        lay = qo.layout(oc, ic, k, 4, 128)
        codes, scales, zeros = synth.make_codes(oc, lay["kq"], lay["n_groups"], 4, seed)
        weak = np.ascontiguousarray(synth.make_weight(oc, ic, seed)[:, ic - k:])
        w64 = qo.dequantize(codes, scales, zeros, weak, 128)
        dy = synth.make_grad_output(m, oc, seed=m)
        ref = qo.linear_bwd_dx(w64, dy)
        w16 = w64.astype(np.float32).astype(np.float16).astype(np.float64)
        rounded = qo.round_fp16(qo.linear_bwd_dx(w16, dy)).astype(np.float64)
        unrounded = qo.round_fp16(ref).astype(np.float64)
        assert worst(rounded, ref) > 1.0
        assert worst(unrounded, ref) < 0.25
        assert np.linalg.norm(rounded - ref) / np.linalg.norm(ref) < 5e-4

