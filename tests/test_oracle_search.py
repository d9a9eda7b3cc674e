"""Pins for the oracle's grid-search quantizer (Sec. 3.1), no GPU.

Pinned against: the plain min-max quantizer (candidate 0 is exactly it; the search can only lower
every group's squared error), a brute-force search written independently with Python floats on
cases whose arithmetic is exact, a hand-made group where truncation must win, and the invariants
of the stored form.
"""
import numpy as np
import pytest

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import synth


def _group_errors(w, codes, scales, zeros, g):
    """Squared error per (row, group) in float64, from the returned stored form only."""
    oc, kq = codes.shape
    ng = scales.shape[1]
    wq = qo.dequantize(codes, scales, zeros, np.zeros((oc, 0), dtype=np.float16), g)
    d = (w[:, :kq].astype(np.float64) - wq) ** 2
    return np.stack([d[:, gi * g:min((gi + 1) * g, kq)].sum(axis=1) for gi in range(ng)], axis=1)


@pytest.mark.parametrize("bits,g,kq,k", [(4, 128, 512, 8), (4, 128, 504, 8), (3, 64, 256, 0), (4, 32, 96, 16)])
def test_one_candidate_is_plain_min_max(bits, g, kq, k):
    w = synth.make_weight(12, kq + k, seed=bits * 100 + g)
    a = qo.quantize_search(w, k, bits, g, 1, 0.01)
    b = qo.quantize_rtn(w, k, bits, g)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint8) if x.dtype != np.uint8 else x, y.view(np.uint8) if y.dtype != np.uint8 else y)


@pytest.mark.parametrize("bits,g,kq,k", [(4, 128, 512, 8), (4, 128, 504, 8), (3, 64, 256, 0), (4, 32, 96, 16)])
def test_search_never_loses_to_min_max_in_any_group(bits, g, kq, k):
    w = synth.make_weight(24, kq + k, seed=7 + bits + g)
    w[3, 5] = np.float16(0.4)          # outliers: truncation pays off here
    w[4, 77] = np.float16(-0.5)
    cs, ss, zs, _ = qo.quantize_search(w, k, bits, g, 80, 0.01)
    cr, sr, zr, _ = qo.quantize_rtn(w, k, bits, g)
    es, er = _group_errors(w, cs, ss, zs, g), _group_errors(w, cr, sr, zr, g)
    assert np.all(es <= er * (1 + 1e-6) + 1e-12)
    assert es[3, 0] < er[3, 0] and es[4, 0] < er[4, 0]    # the groups with an outlier really improved
    assert np.sum(es < er) > es.size // 4                  # and so did many ordinary ones
    # invariants of the stored form
    qmax = (1 << bits) - 1
    assert cs.max() <= qmax and np.all(zs.astype(np.float32) == np.rint(zs.astype(np.float32)))
    assert np.all((zs >= 0) & (zs <= qmax)) and np.all(ss > 0)


def test_hand_made_group_where_truncation_wins():
    # 127 values on the lattice k / 8 (k = 0 .. 7) and one value at 1.0.  Min-max spreads its 16
    # levels over [0, 1] in steps of 1 / 15, which misses the lattice; the range shrunk by 0.9375
    # has steps of exactly 1 / 16 and loses only (1 - 0.9375)^2 on the largest value.
    g, bits = 128, 4
    w = np.zeros((1, g), dtype=np.float16)
    w[0, :127] = (np.arange(127) % 8).astype(np.float16) * np.float16(0.125)    # 0 .. 0.875
    w[0, 127] = np.float16(1.0)
    codes, scales, zeros, _ = qo.quantize_search(w, 0, bits, g, 80, 0.0125)
    rc, rs, rz, _ = qo.quantize_rtn(w, 0, bits, g)
    assert float(rs[0, 0]) == float(np.float16(1.0 / 15.0))
    assert float(scales[0, 0]) == 0.0625 and float(zeros[0, 0]) == 0.0
    assert codes[0, :127].tolist() == [2 * (i % 8) for i in range(127)] and codes[0, 127] == 15
    e_s = _group_errors(w, codes, scales, zeros, g)[0, 0]
    e_r = _group_errors(w, rc, rs, rz, g)[0, 0]
    assert e_s == (1.0 - 0.9375) ** 2 and e_r > 5 * e_s


def _brute(w_row, bits, n_grid, step):
    """Independent search for ONE group of one row, Python floats; valid when all the arithmetic
    involved is exact in float32 (dyadic inputs, power-of-two steps)."""
    qmax = (1 << bits) - 1
    lo0, hi0 = min(0.0, min(w_row)), max(0.0, max(w_row))
    best = None
    for i in range(n_grid):
        p = 1.0 - i * step
        lo, hi = p * lo0, p * hi0
        s = float(np.float16((hi - lo) / qmax))
        if hi == lo:
            s, z = 1.0, 0.0
        else:
            z = min(max(float(np.rint(-lo / s)), 0.0), qmax)
        e = 0.0
        qs = []
        for v in w_row:
            q = min(max(float(np.rint(v / s)) + z, 0.0), qmax)
            qs.append(int(q))
            e += (v - s * (q - z)) ** 2
        if best is None or e < best[0]:
            best = (e, s, z, qs)
    return best


def test_against_independent_brute_force_on_exact_cases():
    r = np.random.default_rng(3)
    g, bits = 32, 4
    # dyadic weights (multiples of 1/64 below 4): with step 1/8 and qmax 15 the candidate ranges are
    # dyadic too; (hi - lo) / 15 is not, but its float16 rounding is what both sides use
    w = (r.integers(-128, 128, size=(6, g)) / 64.0).astype(np.float16)
    codes, scales, zeros, _ = qo.quantize_search(w, 0, bits, g, 6, 0.125)
    for o in range(6):
        e, s, z, qs = _brute([float(v) for v in w[o]], bits, 6, 0.125)
        assert float(scales[o, 0]) == s and float(zeros[o, 0]) == z and codes[o].tolist() == qs


def test_candidates_are_scored_in_plain_float64_and_any_shape_is_taken():
    """search_candidates against a per-element Python-float recomputation from its own (s, z), on a shape
    with a ragged last group and a group size that is no multiple of 8; quantize_search picks the
    first minimum of those scores."""
    r = np.random.default_rng(9)
    oc, kq, k, g, bits, n_grid, step = 3, 27, 2, 12, 3, 7, 0.0625
    w = (r.standard_normal((oc, kq + k)) * 0.05).astype(np.float16)
    s_all, z_all, e_all = qo.search_candidates(w, k, bits, g, n_grid, step)
    assert s_all.shape == (n_grid, oc, 3)
    for i in range(n_grid):
        codes = qo.codes_for_params(w, k, bits, g, s_all[i], z_all[i])
        for o in range(oc):
            for gi in range(3):
                e = 0.0
                for j in range(gi * g, min((gi + 1) * g, kq)):
                    e += (float(w[o, j]) - float(s_all[i, o, gi]) * (int(codes[o, j]) - float(z_all[i, o, gi]))) ** 2
                assert abs(e - e_all[i, o, gi]) <= 1e-12 * max(e, 1e-30)
    codes, scales, zeros, weak = qo.quantize_search(w, k, bits, g, n_grid, step)
    best = np.argmin(e_all, axis=0)
    for o in range(oc):
        for gi in range(3):
            assert scales[o, gi] == s_all[best[o, gi], o, gi] and float(zeros[o, gi]) == z_all[best[o, gi], o, gi]
            assert np.all(e_all[:best[o, gi], o, gi] > e_all[best[o, gi], o, gi])      # the first minimum
    assert np.array_equal(codes, qo.codes_for_params(w, k, bits, g, scales, zeros))
    assert np.array_equal(weak, w[:, kq:])
