"""Pins for the oracle's global weak-column selection and offline reordering (Sec. 3.2, App. B).  No GPU.

Pinned against closed forms, hand-worked votes, planted outlier channels that must be recovered,
scale invariance of a layer's vote, and the invariance of the layer's output under the reordering
(checked with a plain product on other code)."""
import numpy as np
import torch

from oracle import qeft_oracle as qo


def test_sensitivity_closed_forms():
    # every token equal to c: s_j = 2 * (tokens / n_batch) * c_j^2
    c = np.array([1.0, -2.0, 0.5, 0.0], dtype=np.float16)
    x = np.tile(c, (12, 1))
    assert qo.sensitivity(x, 3).tolist() == [2 * 4 * 1.0, 2 * 4 * 4.0, 2 * 4 * 0.25, 0.0]
    # equals the diagonal of the batch-averaged 2 X^T X computed as a matrix on other code
    r = np.random.default_rng(0)
    x = r.standard_normal((6 * 5, 9)).astype(np.float16)
    xt = torch.from_numpy(x).double().reshape(6, 5, 9)
    H = (2 * xt.transpose(1, 2) @ xt).mean(dim=0)
    np.testing.assert_allclose(qo.sensitivity(x, 6), torch.diagonal(H).numpy(), rtol=1e-12)


def test_top_k_order_and_ties():
    assert qo.top_k(np.array([1.0, 5.0, 3.0, 5.0, 0.0]), 3).tolist() == [1, 3, 2]
    assert qo.top_k(np.array([2.0, 2.0, 2.0]), 2).tolist() == [0, 1]
    assert qo.top_k(np.array([1.0, 9.0]), 0).tolist() == []


def test_vote_by_hand():
    s_global = np.zeros(4)
    ids = qo.vote(np.array([8.0, 2.0, 4.0, 2.0]), 2, s_global)     # mean 4: channels 0 and 2 add 2 and 1
    assert ids.tolist() == [0, 2] and s_global.tolist() == [2.0, 0.0, 1.0, 0.0]
    qo.vote(np.array([1.0, 1.0, 1.0, 5.0]), 2, s_global)           # mean 2: channels 3 and 0 add 2.5 and 0.5
    assert s_global.tolist() == [2.5, 0.0, 1.0, 2.5]
    assert qo.top_k(s_global, 2).tolist() == [0, 3]                # tie: lower index first


def test_planted_outlier_channels_are_recovered_and_scale_does_not_matter():
    r = np.random.default_rng(1)
    d, k, planted = 96, 4, [7, 40, 41, 90]
    layers = []
    for li in range(5):
        x = r.standard_normal((64, d)).astype(np.float32)
        x[:, planted] *= 12.0
        if li == 2:
            x[:, 13] *= 30.0           # one layer has an outlier of its own: it gets one vote, not five
        layers.append((x.astype(np.float16), 4))
    got = qo.global_weak_columns(layers, k)
    assert sorted(got.tolist()) == planted
    # a layer's vote is relative to its own mean: rescaling one layer's input changes nothing
    scaled = [(x * np.float16(0.125) if i == 1 else x, b) for i, (x, b) in enumerate(layers)]
    assert qo.global_weak_columns(scaled, k).tolist() == got.tolist()


def test_output_is_invariant_under_the_reordering():
    r = np.random.default_rng(2)
    oc, d, m = 5, 12, 3
    w = r.standard_normal((oc, d))
    x = r.standard_normal((m, d))
    perm = qo.stored_order(d, [9, 2, 5])
    wr, xr = qo.reorder(w, perm, axis=1), qo.reorder(x, perm, axis=1)
    assert wr[:, -3:].tolist() == w[:, [9, 2, 5]].tolist()          # the weak channels end up last, in order
    y = (torch.from_numpy(x) @ torch.from_numpy(w).T).numpy()
    np.testing.assert_allclose(qo.linear_fwd(wr, xr), y, rtol=1e-12, atol=1e-12)
    # a layer that WRITES the hidden state is reordered along its rows: its output comes out reordered
    v = r.standard_normal((d, 7))
    h = r.standard_normal((m, 7))
    np.testing.assert_allclose(qo.linear_fwd(qo.reorder(v, perm, axis=0), h), qo.reorder(h @ v.T, perm, axis=1), rtol=1e-12)


def test_merge_weak_by_hand_and_consistency():
    from fractions import Fraction
    base = np.array([[1.0, 2.0], [0.5, -1.0]], dtype=np.float16)
    tuned = np.array([[1.5, 2.0], [0.25, 1.0]], dtype=np.float16)           # Delta = [[0.5, 0], [-0.25, 2]]
    target = np.array([[10, 20, 30, 40], [1, 2, 3, 4]], dtype=np.float16)
    got = qo.merge_weak(target, tuned, base, idx=[3, 0])                     # weak columns 3 and 0 of the target
    assert got.tolist() == [[10.0, 20.0, 30.0, 40.5], [3.0, 2.0, 3.0, 3.75]]
    assert target.tolist() == [[10, 20, 30, 40], [1, 2, 3, 4]]               # input untouched
    blk = np.array([[7.0, 8.0], [9.0, 10.0]], dtype=np.float16)
    assert qo.merge_weak(blk, tuned, base).tolist() == [[7.5, 8.0], [8.75, 12.0]]   # the target's own weak block
    # merging into a full-precision target at idx, then taking its weak columns, equals merging into the block
    r = np.random.default_rng(4)
    t = r.standard_normal((6, 20)).astype(np.float16)
    a0, a1 = r.standard_normal((6, 5)).astype(np.float16), r.standard_normal((6, 5)).astype(np.float16)
    idx = [17, 3, 4, 11, 0]
    full = qo.merge_weak(t, a1, a0, idx)
    assert np.array_equal(full[:, idx], qo.merge_weak(t[:, idx], a1, a0))
    untouched = [c for c in range(20) if c not in idx]
    assert np.array_equal(full[:, untouched], t[:, untouched])
    # each element is the correctly rounded fp16 of the exact sum when that sum is exact in float32
    o, c = 2, 1
    exact = Fraction(float(t[o, idx[c]])) + Fraction(float(a1[o, c])) - Fraction(float(a0[o, c]))
    assert abs(Fraction(float(full[o, idx[c]])) - exact) <= abs(exact) * Fraction(1, 2048) + Fraction(1, 2 ** 24)
