"""The C-ABI library loads, exports every symbol include/qeft.h declares, and rejects bad
arguments before touching the GPU (no GPU needed: every call here fails validation or is
host-only)."""
import ctypes as C
import os
import re

import pytest

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "qeft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qeft_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared_functions()
    assert names == sorted(B.EXPORTS), "binding and header disagree"
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    for n in ("qeft_pack", "qeft_linear_fwd", "qeft_linear_bwd_dx", "qeft_weak_grad"):   # the four named calls
        assert n in names


@pytest.mark.parametrize("shape", [(512, 512, 8, 4), (4096, 11008, 128, 4), (5120, 13824, 128, 3), (7, 32, 32, 4), (3, 9, 0, 3)])
def test_layout_matches_oracle(shape):
    oc, ic, k, bits = shape
    lay = B.qeft_layout(B.make_desc(oc, ic, k, bits, 128))
    ref = qo.layout(oc, ic, k, bits, 128)
    for f in ("kq", "n_groups", "words_per_row", "row_stride_words", "group_stride", "qweight_bytes", "scales_bytes", "zeros_bytes", "weak_bytes"):
        assert getattr(lay, f) == ref[f], f


def _w(q=0x1000, s=0x2000, z=0x3000, k=0x4000):
    return B.qeft_weight_t(q, s, z, k)


def test_status_strings():
    for st in range(0, -8, -1):
        assert B.raw.qeft_status_string(st) not in (None, b"unknown status")
    assert B.raw.qeft_status_string(-99) == b"unknown status"


def test_descriptor_validation():
    lay = B.qeft_layout_t()
    assert B.raw.qeft_layout(None, C.byref(lay)) == B.QEFT_ERR_NULL
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 5)), C.byref(lay)) == B.QEFT_ERR_BITS
    assert B.raw.qeft_layout(C.byref(B.make_desc(0, 8, 0, 4)), C.byref(lay)) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 9, 4)), C.byref(lay)) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, -1, 4)), C.byref(lay)) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 4, 0)), C.byref(lay)) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 4, 128, 7)), C.byref(lay)) == B.QEFT_ERR_UNSUPPORTED
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 4)), None) == B.QEFT_ERR_NULL
    # the dense layout exists for 3-bit codes only
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 4, 128, B.QEFT_LAYOUT_DENSE3)), C.byref(lay)) == B.QEFT_ERR_UNSUPPORTED
    assert B.raw.qeft_layout(C.byref(B.make_desc(8, 8, 0, 3, 128, B.QEFT_LAYOUT_DENSE3)), C.byref(lay)) == B.QEFT_OK


@pytest.mark.parametrize("oc,ic,k", [(4096, 4096, 128), (13824, 5120, 128), (5120, 13824, 128), (33, 200, 24), (7, 11, 0)])
def test_dense3_layout_matches_oracle(oc, ic, k):
    lay = B.qeft_layout(B.make_desc(oc, ic, k, 3, 128, B.QEFT_LAYOUT_DENSE3))
    ref = qo.layout(oc, ic, k, 3, 128, dense=True)
    assert lay.kq == ref["kq"] and lay.n_groups == ref["n_groups"]
    assert lay.words_per_row == ref["words_per_row"] == (3 * (ic - k) + 31) // 32
    assert lay.row_stride_words == ref["row_stride_words"]
    assert lay.qweight_bytes == ref["qweight_bytes"] and lay.scales_bytes == ref["scales_bytes"]


def test_forward_and_backward_validation():
    d = B.make_desc(64, 256, 128, 4)
    w = _w()
    fwd, dx = B.raw.qeft_linear_fwd, B.raw.qeft_linear_bwd_dx
    X, Y = 0x10000, 0x20000
    assert fwd(C.byref(d), None, X, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_NULL
    assert fwd(C.byref(d), C.byref(_w(q=None)), X, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_NULL
    assert fwd(C.byref(d), C.byref(_w(k=None)), X, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_NULL
    assert fwd(C.byref(d), C.byref(_w(s=0x2002)), X, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_ALIGN
    assert fwd(C.byref(d), C.byref(w), None, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_NULL
    assert fwd(C.byref(d), C.byref(w), X, -1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_SHAPE
    assert fwd(C.byref(d), C.byref(w), X, 1, 248, Y, 64, None, 0, None) == B.QEFT_ERR_SHAPE      # ldx < IC
    assert fwd(C.byref(d), C.byref(w), X, 1, 260, Y, 64, None, 0, None) == B.QEFT_ERR_ALIGN      # ldx % 8
    assert fwd(C.byref(d), C.byref(w), X + 2, 1, 256, Y, 64, None, 0, None) == B.QEFT_ERR_ALIGN
    assert fwd(C.byref(d), C.byref(w), X, 1, 256, Y, 56, None, 0, None) == B.QEFT_ERR_SHAPE      # ldy < OC
    assert fwd(C.byref(d), C.byref(w), X, 0, 256, Y, 64, None, 0, None) == B.QEFT_OK             # M = 0: no-op
    assert fwd(C.byref(d), C.byref(w), None, 0, 0, None, 0, None, 0, None) == B.QEFT_OK
    assert dx(C.byref(d), C.byref(w), X, 2, 56, Y, 256, None, 0, None) == B.QEFT_ERR_SHAPE       # lddy < OC
    assert dx(C.byref(d), C.byref(w), X, 2, 64, Y, 248, None, 0, None) == B.QEFT_ERR_SHAPE       # lddx < IC
    assert dx(C.byref(d), C.byref(w), X, 2, 64, None, 256, None, 0, None) == B.QEFT_ERR_NULL
    assert dx(C.byref(d), C.byref(w), X, 0, 64, Y, 256, None, 0, None) == B.QEFT_OK
    # all-weak layer: the quantized pointers may be NULL
    d2 = B.make_desc(64, 128, 128, 4)
    assert fwd(C.byref(d2), C.byref(_w(q=None, s=None, z=None)), X, 0, 128, Y, 64, None, 0, None) == B.QEFT_OK
    d3 = B.make_desc(64, 128, 0, 3)
    assert fwd(C.byref(d3), C.byref(_w(k=None)), X, 0, 128, Y, 64, None, 0, None) == B.QEFT_OK


def test_three_bit_workspace_rules():
    """3-bit layers at M > 16 may take an fp16 copy in a caller workspace: its size, and the errors that
    precede any launch (too small, misaligned)."""
    fwd, dx = B.raw.qeft_linear_fwd, B.raw.qeft_linear_bwd_dx
    X, Y, WS = 0x10000, 0x200000, 0x4000000
    for layout in (B.QEFT_LAYOUT_CANONICAL, B.QEFT_LAYOUT_DENSE3):
        d = B.make_desc(64, 256, 128, 3, 128, layout)
        need = 64 * 256 * 2
        assert B.qeft_workspace_bytes(d, B.QEFT_OP_FWD, 17) == need == B.qeft_workspace_bytes(d, B.QEFT_OP_BWD_DX, 4096)
        assert B.qeft_workspace_bytes(d, B.QEFT_OP_FWD, 16) == 0          # decode sizes use no copy
        assert fwd(C.byref(d), C.byref(_w()), X, 32, 256, Y, 64, WS, need - 2, None) == B.QEFT_ERR_WORKSPACE
        assert fwd(C.byref(d), C.byref(_w()), X, 32, 256, Y, 64, WS + 8, need, None) == B.QEFT_ERR_ALIGN
        assert dx(C.byref(d), C.byref(_w()), X, 32, 64, Y, 256, WS, need - 2, None) == B.QEFT_ERR_WORKSPACE
        assert dx(C.byref(d), C.byref(_w()), X, 32, 64, Y, 256, WS + 8, need, None) == B.QEFT_ERR_ALIGN
    assert B.qeft_workspace_bytes(B.make_desc(64, 256, 128, 4), B.QEFT_OP_FWD, 4096) == 0       # 4-bit layers never take a copy
    assert B.qeft_workspace_bytes(B.make_desc(64, 256, 256, 3), B.QEFT_OP_FWD, 4096) == 0       # nothing quantized
    assert B.qeft_workspace_bytes(B.make_desc(64, 260, 128, 3), B.QEFT_OP_FWD, 4096) == 0       # IC not a multiple of 8: general kernel


def test_last_round_split_workspace_rules():
    """Launches of 160 tiles or more: only the tiles of a sparsely filled last round are split (per XCD: the tiles past its
    last multiple of 32, when at most 16), each partial tile a 128 KiB slot; launches that fill their rounds need nothing."""
    slot = 256 * 256 * 2

    def slots(oc, ic, k, m, op):
        return B.qeft_workspace_bytes(B.make_desc(oc, ic, k, 4), op, m) / slot

    F, D = B.QEFT_OP_FWD, B.QEFT_OP_BWD_DX
    # 13B, M = 4096: 20 x 16 = 320 tiles -> 8 per XCD in the last round, 4 splits; 54 x 16 = 864 -> 12 per XCD, 2 splits
    assert slots(5120, 5120, 128, 4096, F) == 64 * 4 and slots(5120, 5120, 128, 4096, D) == 64 * 4
    assert slots(13824, 5120, 128, 4096, F) == 96 * 2 and slots(13824, 5120, 128, 4096, D) == 64 * 4
    assert slots(5120, 13824, 128, 4096, F) == 64 * 4 and slots(5120, 13824, 128, 4096, D) == 96 * 2
    # 70B, M = 2048: 112 x 8 = 896 tiles -> 16 per XCD, 2 splits; 32 x 8 = 256 tiles fill one round exactly
    assert slots(28672, 8192, 256, 2048, F) == 128 * 2 and slots(28672, 8192, 256, 2048, D) == 0
    assert slots(8192, 28672, 256, 2048, D) == 128 * 2 and slots(8192, 28672, 256, 2048, F) == 0
    # 7B, M = 4096: 256 tiles, or 688 = 86 per XCD with 22 in the last round (more than half of the CUs): no split
    for oc, ic in ((4096, 4096), (11008, 4096), (4096, 11008)):
        assert slots(oc, ic, 128, 4096, F) == 0 and slots(oc, ic, 128, 4096, D) == 0
    # a short contraction does not pay for the second pass: 264 tiles, 16 stages against 32
    assert slots(8448, 1024 + 128, 128, 2048, F) == 0 and slots(8448, 2048 + 128, 128, 2048, F) == 8 * 4


def test_forward_k_split_workspace_rules():
    """4-bit forward launches with few output tiles may split K over an optional workspace of fp16 partial tiles."""
    fwd = B.raw.qeft_linear_fwd
    X, Y, WS = 0x10000, 0x2000000, 0x40000000
    d = B.make_desc(1024, 8192, 256, 4)                      # 4 x 8 tiles at M = 2048, 124 quantized stages: 8 splits of 16
    need = B.qeft_workspace_bytes(d, B.QEFT_OP_FWD, 2048)
    assert need == 8 * 2048 * 1024 * 2
    assert B.qeft_workspace_bytes(d, B.QEFT_OP_BWD_DX, 2048) == 0                                # 32 x 8 tiles: no split
    d4 = B.make_desc(4096, 4096, 128, 4)                     # input gradient at M = 256: 16 tiles, 64 stages of rows: 8 splits
    need_dx = B.qeft_workspace_bytes(d4, B.QEFT_OP_BWD_DX, 256)
    assert need_dx == 8 * 256 * 4096 * 2
    assert B.raw.qeft_linear_bwd_dx(C.byref(d4), C.byref(_w()), X, 256, 4096, Y, 4096, WS, need_dx - 2, None) == B.QEFT_ERR_WORKSPACE
    assert B.raw.qeft_linear_bwd_dx(C.byref(d4), C.byref(_w()), X, 256, 4096, Y, 4096, WS + 8, need_dx, None) == B.QEFT_ERR_ALIGN
    assert B.qeft_workspace_bytes(d, B.QEFT_OP_FWD, 16) == 0                                    # decode sizes
    assert B.qeft_workspace_bytes(B.make_desc(4096, 4096, 128, 4), B.QEFT_OP_FWD, 4096) == 0     # 256 tiles: no split
    assert B.qeft_workspace_bytes(B.make_desc(4096, 4096, 128, 4), B.QEFT_OP_FWD, 256) == 4 * 256 * 4096 * 2 * 2   # 16 tiles, 62 stages: 7 chunks -> 8 splits
    assert fwd(C.byref(d), C.byref(_w()), X, 2048, 8192, Y, 1024, WS, need - 2, None) == B.QEFT_ERR_WORKSPACE
    assert fwd(C.byref(d), C.byref(_w()), X, 2048, 8192, Y, 1024, WS + 8, need, None) == B.QEFT_ERR_ALIGN


def test_forward_group_validation():
    grp = B.raw.qeft_linear_fwd_group
    X = 0x10000
    d = B.make_desc(64, 256, 128, 4)
    descs = (B.qeft_desc_t * 2)(d, B.make_desc(32, 256, 128, 4))
    ws = (B.qeft_weight_t * 2)(_w(), _w())
    ys = (C.c_void_p * 2)(0x20000, 0x30000)
    ldy = (C.c_int64 * 2)(64, 32)
    assert grp(2, descs, ws, X, 0, 256, ys, ldy, None) == B.QEFT_OK                 # M = 0: no-op
    assert grp(0, descs, ws, X, 0, 256, ys, ldy, None) == B.QEFT_ERR_SHAPE
    assert grp(5, descs, ws, X, 0, 256, ys, ldy, None) == B.QEFT_ERR_SHAPE
    assert grp(2, None, ws, X, 0, 256, ys, ldy, None) == B.QEFT_ERR_NULL
    assert grp(2, descs, ws, X, 0, 256, None, ldy, None) == B.QEFT_ERR_NULL
    assert grp(2, descs, ws, X, 1, 248, ys, ldy, None) == B.QEFT_ERR_SHAPE          # ldx < IC
    assert grp(2, descs, ws, X, 1, 256, ys, (C.c_int64 * 2)(64, 24), None) == B.QEFT_ERR_SHAPE   # ldy[1] < OC
    # the layers of a group share the input: in_features, n_weak, bits and group size must agree
    for other in (B.make_desc(32, 512, 128, 4), B.make_desc(32, 256, 64, 4), B.make_desc(32, 256, 128, 3),
                  B.make_desc(32, 256, 128, 4, 64)):
        bad = (B.qeft_desc_t * 2)(d, other)
        assert grp(2, bad, ws, X, 0, 256, ys, ldy, None) == B.QEFT_ERR_SHAPE


def test_irregular_validation():
    d = B.make_desc(64, 256, 128, 4)
    w = _w()
    fwd, dx = B.raw.qeft_linear_fwd_irregular, B.raw.qeft_linear_bwd_dx_irregular
    X, Y, P, WS = 0x10000, 0x20000, 0x30000, 0x40000
    M = 6    # more rows than the decode kernel gathers in place: the workspace is required
    need = B.qeft_workspace_bytes(d, B.QEFT_OP_FWD_IRREGULAR, M)
    assert need == M * 256 * 2 and B.qeft_workspace_bytes(d, B.QEFT_OP_BWD_DX_IRREGULAR, M) == need
    assert B.qeft_workspace_bytes(B.make_desc(64, 333, 21, 4), B.QEFT_OP_FWD_IRREGULAR, 2) == 2 * 336 * 2   # row pitch rounded up to 8
    assert fwd(C.byref(d), C.byref(w), P, X, 0, 256, Y, 64, None, 0, None) == B.QEFT_OK              # M = 0: no-op
    assert fwd(C.byref(d), C.byref(w), None, X, M, 256, Y, 64, WS, need, None) == B.QEFT_ERR_NULL    # no table
    assert fwd(C.byref(d), C.byref(w), P + 4, X, M, 256, Y, 64, WS, need, None) == B.QEFT_ERR_ALIGN
    assert fwd(C.byref(d), C.byref(w), P, X, M, 256, Y, 64, None, 0, None) == B.QEFT_ERR_WORKSPACE
    assert fwd(C.byref(d), C.byref(w), P, X, M, 256, Y, 64, WS, need - 1, None) == B.QEFT_ERR_WORKSPACE
    assert fwd(C.byref(d), C.byref(w), P, X, M, 256, Y, 64, WS + 4, need, None) == B.QEFT_ERR_WORKSPACE
    assert fwd(C.byref(d), C.byref(w), P, X, M, 248, Y, 64, WS, need, None) == B.QEFT_ERR_SHAPE      # ldx < IC
    assert fwd(C.byref(d), C.byref(w), P, X, M, 256, Y, 56, WS, need, None) == B.QEFT_ERR_SHAPE      # ldy < OC
    assert fwd(C.byref(d), C.byref(w), P, X, 2, 256, Y, 56, None, 0, None) == B.QEFT_ERR_SHAPE       # decode-sized: same checks
    assert fwd(C.byref(d), C.byref(_w(q=None)), P, X, M, 256, Y, 64, WS, need, None) == B.QEFT_ERR_NULL
    assert fwd(C.byref(d), C.byref(_w(q=None)), P, X, 2, 256, Y, 64, None, 0, None) == B.QEFT_ERR_NULL
    assert dx(C.byref(d), C.byref(w), P, X, 0, 64, Y, 256, None, 0, None) == B.QEFT_OK
    assert dx(C.byref(d), C.byref(w), None, X, M, 64, Y, 256, WS, need, None) == B.QEFT_ERR_NULL
    assert dx(C.byref(d), C.byref(w), P, X, M, 64, Y, 256, WS, need - 1, None) == B.QEFT_ERR_WORKSPACE
    assert dx(C.byref(d), C.byref(w), P, X, M, 56, Y, 256, WS, need, None) == B.QEFT_ERR_SHAPE       # lddy < OC
    assert dx(C.byref(d), C.byref(w), P, X, M, 64, Y, 248, WS, need, None) == B.QEFT_ERR_SHAPE       # lddx < IC


def test_reordering_validation():
    R = B.raw
    X, O, P, WS = 0x10000, 0x20000, 0x30000, 0x40000
    assert R.qeft_sensitivity_workspace(4096, 1000) > 0 and R.qeft_sensitivity_workspace(0, 5) == 0
    need = R.qeft_sensitivity_workspace(96, 64)
    assert R.qeft_sensitivity(X, 64, 96, 100, 4, O, WS, need, None) == B.QEFT_ERR_SHAPE          # d % 8
    assert R.qeft_sensitivity(X, 64, 88, 96, 4, O, WS, need, None) == B.QEFT_ERR_SHAPE           # ldx < d
    assert R.qeft_sensitivity(X, 64, 96, 96, 0, O, WS, need, None) == B.QEFT_ERR_SHAPE           # n_batch
    assert R.qeft_sensitivity(None, 64, 96, 96, 4, O, WS, need, None) == B.QEFT_ERR_NULL
    assert R.qeft_sensitivity(X, 64, 96, 96, 4, None, WS, need, None) == B.QEFT_ERR_NULL
    assert R.qeft_sensitivity(X, 64, 96, 96, 4, O, WS, need - 1, None) == B.QEFT_ERR_WORKSPACE
    assert R.qeft_vote(X, 96, 97, O, None, None) == B.QEFT_ERR_SHAPE                               # k > d
    assert R.qeft_vote(None, 96, 4, O, None, None) == B.QEFT_ERR_NULL
    assert R.qeft_vote(X, 96, 4, None, None, None) == B.QEFT_ERR_NULL
    assert R.qeft_vote(X, 96, 0, None, None, None) == B.QEFT_OK                                    # nothing to select
    assert R.qeft_weak_order(P, 4, 0, O, None) == B.QEFT_ERR_SHAPE
    assert R.qeft_weak_order(None, 4, 96, O, None) == B.QEFT_ERR_NULL
    assert R.qeft_weak_order(P, 4, 96, None, None) == B.QEFT_ERR_NULL
    assert R.qeft_reorder(X, 8, 96, 96, P, 2, O, 96, None) == B.QEFT_ERR_SHAPE                     # axis
    assert R.qeft_reorder(X, 8, 96, 88, P, 1, O, 96, None) == B.QEFT_ERR_SHAPE                     # lda < cols
    assert R.qeft_reorder(X, 8, 96, 96, None, 1, O, 96, None) == B.QEFT_ERR_NULL
    assert R.qeft_reorder(X, 8, 96, 96, P, 1, X, 96, None) == B.QEFT_ERR_SHAPE                     # in place
    assert R.qeft_reorder(X, 8, 100, 104, P, 0, O, 104, None) == B.QEFT_ERR_UNSUPPORTED            # rows of odd width
    assert R.qeft_reorder(X, 0, 96, 96, P, 1, O, 96, None) == B.QEFT_OK


def test_merge_validation():
    mg = B.raw.qeft_merge_weak
    A1, A0, T, P = 0x10000, 0x20000, 0x30000, 0x40000
    assert mg(A1, A0, 8, 4, P, T, 16, 2, None) == B.QEFT_ERR_SHAPE            # fewer target columns than weak ones
    assert mg(A1, A0, 8, 4, P, T, 8, 16, None) == B.QEFT_ERR_SHAPE            # ldt < columns
    assert mg(A1, A0, -1, 4, P, T, 16, 16, None) == B.QEFT_ERR_SHAPE
    assert mg(None, A0, 8, 4, P, T, 16, 16, None) == B.QEFT_ERR_NULL
    assert mg(A1, A0, 8, 4, P, None, 16, 16, None) == B.QEFT_ERR_NULL
    assert mg(A1, A0, 0, 4, P, T, 16, 16, None) == B.QEFT_OK
    assert mg(A1, A0, 8, 0, None, T, 16, 16, None) == B.QEFT_OK


def test_pack_and_weak_grad_validation():
    d = B.make_desc(64, 256, 128, 4)
    w = _w()
    ps = B.raw.qeft_pack_search
    assert ps(C.byref(d), None, 256, 80, 0.01, C.byref(w), None) == B.QEFT_ERR_NULL
    assert ps(C.byref(d), 0x10000, 128, 80, 0.01, C.byref(w), None) == B.QEFT_ERR_SHAPE           # ldw < IC
    assert ps(C.byref(d), 0x10000, 256, 0, 0.01, C.byref(w), None) == B.QEFT_ERR_SHAPE            # no candidate
    assert ps(C.byref(d), 0x10000, 256, 101, 0.01, C.byref(w), None) == B.QEFT_ERR_SHAPE          # range would vanish
    assert ps(C.byref(d), 0x10000, 256, 80, -0.5, C.byref(w), None) == B.QEFT_ERR_SHAPE
    assert ps(C.byref(B.make_desc(64, 256, 128, 4, 100)), 0x10000, 256, 80, 0.01, C.byref(w), None) == B.QEFT_ERR_UNSUPPORTED   # g % 8
    assert ps(C.byref(B.make_desc(64, 256 + 4, 128, 4)), 0x10000, 264, 80, 0.01, C.byref(w), None) == B.QEFT_ERR_UNSUPPORTED  # Kq % 8
    assert B.raw.qeft_pack(C.byref(d), None, 256, C.byref(w), None) == B.QEFT_ERR_NULL
    assert B.raw.qeft_pack(C.byref(d), 0x10000, 128, C.byref(w), None) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_pack(C.byref(d), 0x10000, 256, None, None) == B.QEFT_ERR_NULL
    assert B.raw.qeft_pack_codes(C.byref(d), None, 0x100, 0x200, 0x300, C.byref(w), None) == B.QEFT_ERR_NULL
    wg = B.raw.qeft_weak_grad
    dY, Xw, dW = 0x10000, 0x20000, 0x30000
    assert wg(C.byref(d), dY, 4, 64, Xw, 128, dW, 2, 0, None, 0, None) == B.QEFT_ERR_UNSUPPORTED   # dtype
    assert wg(C.byref(d), None, 4, 64, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert wg(C.byref(d), dY, 4, 64, Xw, 120, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE         # ldxw < k
    assert wg(C.byref(d), dY, 4, 64, Xw, 128, None, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert wg(C.byref(d), dY, 0, 64, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_OK
    assert wg(C.byref(d), dY, -3, 64, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE
    need = B.qeft_workspace_bytes(B.make_desc(4096, 4096, 128, 4), B.QEFT_OP_WEAK_GRAD, 4096)
    if need:
        d4 = B.make_desc(4096, 4096, 128, 4)
        assert wg(C.byref(d4), dY, 4096, 4096, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_WORKSPACE
        assert wg(C.byref(d4), dY, 4096, 4096, Xw, 128, dW, 1, 0, 0x40000, need - 1, None) == B.QEFT_ERR_WORKSPACE
    assert B.qeft_workspace_bytes(d, B.QEFT_OP_FWD, 0) == 0


def test_backward_in_one_call_validation():
    """qeft_linear_bwd: every error comes before a launch, also the weak gradient's when the two steps
    would run one after the other."""
    bw = B.raw.qeft_linear_bwd
    d = B.make_desc(64, 256, 128, 4)
    w = _w()
    dY, dX, Xw, dW, WS = 0x10000, 0x20000, 0x30000, 0x40000, 0x4000000
    assert bw(C.byref(d), None, dY, 4, 64, dX, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 256, Xw, 128, dW, 2, 0, None, 0, None) == B.QEFT_ERR_UNSUPPORTED  # dtype
    assert bw(C.byref(d), C.byref(w), None, 4, 64, dX, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert bw(C.byref(d), C.byref(w), dY, 4, 56, dX, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE       # lddy < OC
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, None, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 248, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE       # lddx < IC
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 256, None, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 256, Xw, 120, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE       # ldxw < k
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 256, Xw, 128, None, 1, 0, None, 0, None) == B.QEFT_ERR_NULL
    assert bw(C.byref(d), C.byref(w), dY, 4, 64, dX, 256, Xw, 128, dW + 4, 1, 0, None, 0, None) == B.QEFT_ERR_ALIGN
    assert bw(C.byref(d), C.byref(w), dY, -1, 64, dX, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_ERR_SHAPE
    assert bw(C.byref(d), C.byref(w), dY, 0, 64, dX, 256, Xw, 128, dW, 1, 0, None, 0, None) == B.QEFT_OK              # M = 0: no-op
    # the weak gradient's workspace is asked for whichever way the two steps run: 11008 x 4096 with 128 weak columns
    # goes out as one launch, 4096 x 8192 with 256 as two
    for oc, ic, k, m in ((11008, 4096, 128, 4096), (4096, 8192, 256, 2048)):
        d4 = B.make_desc(oc, ic, k, 4)
        need = B.qeft_workspace_bytes(d4, B.QEFT_OP_WEAK_GRAD, m)
        assert need > 0
        assert bw(C.byref(d4), C.byref(w), dY, m, oc, dX, ic, Xw, k, dW, 1, 0, None, 0, None) == B.QEFT_ERR_WORKSPACE
        assert bw(C.byref(d4), C.byref(w), dY, m, oc, dX, ic, Xw, k, dW, 1, 0, WS, need - 1, None) == B.QEFT_ERR_WORKSPACE
        assert bw(C.byref(d4), C.byref(w), dY, m, oc, dX, ic, Xw, k, dW, 1, 0, WS + 8, need, None) == B.QEFT_ERR_WORKSPACE
    # QEFT_OP_BWD: the larger of the two steps' amounts (13824 x 5120: the last round's 96 tiles split two ways)
    d5 = B.make_desc(13824, 5120, 128, 4)
    a, b = B.qeft_workspace_bytes(d5, B.QEFT_OP_BWD_DX, 4096), B.qeft_workspace_bytes(d5, B.QEFT_OP_WEAK_GRAD, 4096)
    assert a > 0 and b > 0 and B.qeft_workspace_bytes(d5, B.QEFT_OP_BWD, 4096) == max(a, b)
    d6 = B.make_desc(13824, 5120, 128, 3)      # 3-bit: room for the fp16 copy (and its split), which is the larger amount
    a, b = B.qeft_workspace_bytes(d6, B.QEFT_OP_BWD_DX, 4096), B.qeft_workspace_bytes(d6, B.QEFT_OP_WEAK_GRAD, 4096)
    assert a >= 13824 * 5120 * 2 > b and B.qeft_workspace_bytes(d6, B.QEFT_OP_BWD, 4096) == a


def test_dimension_limits():
    """QEFT_MAX_DIM: larger shapes and row counts are refused before any size arithmetic could overflow (a workspace
    query for 2^40 rows used to end in a division by zero)."""
    lim = 1 << 24
    lay = B.qeft_layout_t()
    assert B.raw.qeft_layout(C.byref(B.make_desc(lim, lim, 128, 4)), C.byref(lay)) == B.QEFT_OK
    assert lay.qweight_bytes == lim * ((lim - 128) // 8) * 4
    for d in (B.make_desc(lim + 8, 4096, 128, 4), B.make_desc(4096, lim + 8, 128, 4), B.make_desc(4096, 4096, 128, 4, lim + 8)):
        assert B.raw.qeft_layout(C.byref(d), C.byref(lay)) == B.QEFT_ERR_SHAPE
        assert B.qeft_workspace_bytes(d, B.QEFT_OP_WEAK_GRAD, 4096) == 0
    d = B.make_desc(4096, 4096, 128, 4)
    for op in (B.QEFT_OP_FWD, B.QEFT_OP_BWD_DX, B.QEFT_OP_WEAK_GRAD, B.QEFT_OP_FWD_IRREGULAR, B.QEFT_OP_BWD):
        assert B.qeft_workspace_bytes(d, op, 1 << 40) == 0
        assert B.qeft_workspace_bytes(d, op, lim + 1) == 0
    assert B.qeft_workspace_bytes(d, B.QEFT_OP_WEAK_GRAD, lim) > 0
    w = _w()
    assert B.raw.qeft_linear_fwd(C.byref(d), C.byref(w), 0x10000, lim + 1, 4096, 0x20000, 4096, None, 0, None) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_linear_bwd_dx(C.byref(d), C.byref(w), 0x10000, 1 << 40, 4096, 0x20000, 4096, None, 0, None) == B.QEFT_ERR_SHAPE
    assert B.raw.qeft_sensitivity_workspace(4096, 1 << 40) == 0 and B.raw.qeft_sensitivity_workspace(lim + 8, 4096) == 0
