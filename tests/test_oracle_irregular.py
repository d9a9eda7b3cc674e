"""Pins for the oracle's irregular-index variant (weak columns left in place, the layout of the
attention output projection, Sec. 3.2 / Limitations).  No GPU.

Pinned against the definition written out independently: rebuild the dense weight in ORIGINAL
channel order with explicit Python loops, then use a plain product (torch CPU, other code) and
exact rationals on tiny cases; plus the reductions and identities a wrong gather / scatter
direction, an off-by-one in the complement or a dropped weak column would break.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo


def _dense_original(w_stored, weak_idx, ic):
    """W in original channel order, column by column, without using the oracle's permutation."""
    oc = w_stored.shape[0]
    k = len(weak_idx)
    W = np.zeros((oc, ic), dtype=np.float64)
    weak_set = {int(c): n for n, c in enumerate(weak_idx)}
    nxt = 0   # next stored quantized column
    for c in range(ic):
        if c in weak_set:
            W[:, c] = w_stored[:, ic - k + weak_set[c]]
        else:
            W[:, c] = w_stored[:, nxt]
            nxt += 1
    assert nxt == ic - k
    return W


CASES = [  # oc, ic, weak_idx, m
    (3, 10, [7, 2], 2),            # order of the weak block follows weak_idx, not the channel order
    (4, 16, [0, 15, 8], 3),        # first and last channel weak
    (2, 9, [], 1),                 # no weak column: identity
    (2, 6, [0, 1, 2, 3, 4, 5], 2),  # every channel weak, in place
    (5, 33, [31, 3, 4, 17], 4),
]


@pytest.mark.parametrize("oc,ic,weak_idx,m", CASES)
def test_irregular_products_equal_the_dense_definition(oc, ic, weak_idx, m):
    r = np.random.default_rng(oc * 100 + ic)
    w_stored = r.standard_normal((oc, ic))
    x = r.standard_normal((m, ic)).astype(np.float16)
    dy = r.standard_normal((m, oc)).astype(np.float16)
    perm = qo.stored_order(ic, weak_idx)
    W = _dense_original(w_stored, weak_idx, ic)
    y_ref = (torch.from_numpy(x).double() @ torch.from_numpy(W).T).numpy()
    dx_ref = (torch.from_numpy(dy).double() @ torch.from_numpy(W)).numpy()
    np.testing.assert_allclose(qo.linear_fwd_irregular(w_stored, perm, x), y_ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(qo.linear_bwd_dx_irregular(w_stored, perm, dy), dx_ref, rtol=1e-12, atol=1e-12)


def test_stored_order_by_hand():
    # channels 0..7, weak 5 and 1 (in that order): complement ascending, then 5, 1
    assert qo.stored_order(8, [5, 1]).tolist() == [0, 2, 3, 4, 6, 7, 5, 1]
    assert qo.stored_order(4, []).tolist() == [0, 1, 2, 3]
    assert qo.stored_order(3, [2, 0, 1]).tolist() == [2, 0, 1]
    p = qo.stored_order(100, [99, 0, 50])
    assert sorted(p.tolist()) == list(range(100)) and p[-3:].tolist() == [99, 0, 50]


def test_contiguous_tail_reduces_to_the_regular_layer():
    # weak columns already at the end, in order: the irregular variant is the regular one
    r = np.random.default_rng(5)
    oc, ic, k, m = 6, 40, 8, 3
    w = r.standard_normal((oc, ic))
    x = r.standard_normal((m, ic)).astype(np.float16)
    dy = r.standard_normal((m, oc)).astype(np.float16)
    perm = qo.stored_order(ic, list(range(ic - k, ic)))
    assert perm.tolist() == list(range(ic))
    # (equal up to the summation order of the library product on a gathered copy)
    np.testing.assert_allclose(qo.linear_fwd_irregular(w, perm, x), qo.linear_fwd(w, x), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(qo.linear_bwd_dx_irregular(w, perm, dy), qo.linear_bwd_dx(w, dy), rtol=1e-13, atol=1e-13)


def test_exact_rational_tiny_case():
    # integers small enough for exact float64, checked with Fractions and explicit indices
    w_stored = np.array([[1, 2, 3, 4], [5, 6, 7, 8]], dtype=np.float64)   # stored order: channels 0, 3 | weak 2, 1
    weak_idx = [2, 1]
    x = np.array([[1, 10, 100, 1000]], dtype=np.float16)                  # original order
    perm = qo.stored_order(4, weak_idx)
    assert perm.tolist() == [0, 3, 2, 1]
    y = qo.linear_fwd_irregular(w_stored, perm, x)
    # row 0: 1*x0 + 2*x3 + 3*x2 + 4*x1
    assert Fraction(float(y[0, 0])) == 1 * 1 + 2 * 1000 + 3 * 100 + 4 * 10
    assert Fraction(float(y[0, 1])) == 5 * 1 + 6 * 1000 + 7 * 100 + 8 * 10
    dy = np.array([[1, 2]], dtype=np.float16)
    dx = qo.linear_bwd_dx_irregular(w_stored, perm, dy)
    # dX[c] = sum_o dy[o] W[o][c]; channel 0 <- stored 0, 1 <- stored 3, 2 <- stored 2, 3 <- stored 1
    assert dx[0].tolist() == [1 + 10, 4 + 16, 3 + 14, 2 + 12]


def test_adjoint_identity():
    r = np.random.default_rng(9)
    oc, ic, m = 7, 29, 5
    w = r.standard_normal((oc, ic))
    perm = qo.stored_order(ic, [4, 28, 11, 0, 19])
    x = r.standard_normal((m, ic)).astype(np.float16)
    dy = r.standard_normal((m, oc)).astype(np.float16)
    lhs = np.sum(qo.linear_fwd_irregular(w, perm, x) * dy.astype(np.float64))
    rhs = np.sum(qo.linear_bwd_dx_irregular(w, perm, dy) * x.astype(np.float64))
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))
