"""Pins for the oracle's layout calculator and bit packing (no GPU)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import qeft_oracle as qo


# ---- hand-written bit patterns: code i of a word sits at bit bits*i ----------------
def test_pack4_literal_words():
    codes = np.array([[0, 1, 2, 3, 4, 5, 6, 7, 15, 0, 0, 0, 0, 0, 0, 8, 9]], dtype=np.uint8)
    w = qo.pack_codes(codes, 4, 4)
    assert w.dtype == np.uint32 and w.shape == (1, 4)
    assert [int(v) for v in w[0]] == [0x76543210, 0x8000000F, 0x00000009, 0]


def test_pack3_literal_words():
    # ten 3-bit codes per word, bits 30..31 stay zero
    codes = np.array([[1, 2, 3, 4, 5, 6, 7, 0, 1, 7, 5]], dtype=np.uint8)
    w = qo.pack_codes(codes, 3, 4)
    first = (1 | 2 << 3 | 3 << 6 | 4 << 9 | 5 << 12 | 6 << 15 | 7 << 18 | 0 << 21 | 1 << 24 | 7 << 27)
    assert first == 0o7_1_0_7_6_5_4_3_2_1          # octal digits are the codes, last first
    assert [int(v) for v in w[0]] == [first, 5, 0, 0]
    assert all(int(v) >> 30 == 0 for v in w[0])


def test_unpack_literal():
    w = np.array([[0xFEDCBA98, 0x00000021, 0, 0]], dtype=np.uint32)
    assert qo.unpack_codes(w, 10, 4).tolist() == [[8, 9, 10, 11, 12, 13, 14, 15, 1, 2]]
    w3 = np.array([[0o1234567012, 0o3, 0, 0]], dtype=np.uint32)
    assert qo.unpack_codes(w3, 11, 3).tolist() == [[2, 1, 0, 7, 6, 5, 4, 3, 2, 1, 3]]


@settings(max_examples=60, deadline=None)
@given(bits=st.sampled_from([3, 4]), oc=st.integers(1, 5), kq=st.integers(0, 97), seed=st.integers(0, 2**31))
def test_pack_unpack_roundtrip(bits, oc, kq, seed):
    r = np.random.default_rng(seed)
    codes = r.integers(0, 1 << bits, size=(oc, kq), dtype=np.uint8)
    lay = qo.layout(oc, kq + 3, 3, bits, 16)
    w = qo.pack_codes(codes, bits, lay["row_stride_words"])
    assert np.array_equal(qo.unpack_codes(w, kq, bits), codes)
    # padding words and unused bits are zero: re-packing the unpacked codes is the identity
    assert w[:, lay["words_per_row"]:].sum() == 0
    if bits == 3:
        assert (w >> np.uint32(30)).sum() == 0
    # every code is recoverable by plain integer arithmetic on Python ints
    per = 8 if bits == 4 else 10
    for o in range(oc):
        for j in range(kq):
            assert (int(w[o, j // per]) >> (bits * (j % per))) & ((1 << bits) - 1) == int(codes[o, j])


def test_pack_rejects_out_of_range():
    with pytest.raises(ValueError):
        qo.pack_codes(np.array([[8]], dtype=np.uint8), 3, 4)


# ---- layout closed forms ------------------------------------------------------------
# (OC, IC, k, bits) -> (Kq, G, words per row, stride, total stored bytes), worked by hand
LAYOUT_CASES = [
    ((512, 512, 8, 4), (504, 4, 63, 64, 155648)),
    ((4096, 4096, 128, 4), (3968, 31, 496, 496, 9699328)),
    ((11008, 4096, 128, 4), (3968, 31, 496, 496, 26066944)),
    ((4096, 11008, 128, 4), (10880, 85, 1360, 1360, 24772608)),
    ((5120, 5120, 128, 3), (4992, 39, 500, 512, 12615680)),
    ((5120, 13824, 128, 3), (13696, 107, 1370, 1376, 31784960)),
    ((5120, 13824, 128, 4), (13696, 107, 1712, 1712, 38666240)),
    ((28672, 8192, 256, 4), (7936, 62, 992, 992, 135790592)),
    ((8192, 28672, 256, 4), (28416, 222, 3552, 3552, 127926272)),
]


@pytest.mark.parametrize("shape,expect", LAYOUT_CASES)
def test_layout_closed_form(shape, expect):
    oc, ic, k, bits = shape
    lay = qo.layout(oc, ic, k, bits, 128)
    total = lay["qweight_bytes"] + lay["scales_bytes"] + lay["zeros_bytes"] + lay["weak_bytes"]
    assert (lay["kq"], lay["n_groups"], lay["words_per_row"], lay["row_stride_words"], total) == expect
    # bytes = OC * (4*stride + 2*Gs + 2*Gs + 2*k) with Gs = G rounded up to a multiple of 8
    gs = -(-expect[1] // 8) * 8
    assert lay["group_stride"] == gs
    assert total == oc * (4 * expect[3] + 4 * gs + 2 * k)


def test_layout_degenerate():
    lay = qo.layout(7, 32, 32, 4, 128)          # every column weak: nothing quantized
    assert (lay["kq"], lay["n_groups"], lay["qweight_bytes"], lay["weak_bytes"]) == (0, 0, 0, 7 * 32 * 2)
    lay = qo.layout(7, 32, 0, 3, 128)           # no weak column, one partial group
    assert (lay["kq"], lay["n_groups"], lay["words_per_row"], lay["row_stride_words"], lay["weak_bytes"]) == (32, 1, 4, 16, 0)
    with pytest.raises(ValueError):
        qo.layout(4, 8, 9, 4, 128)
    with pytest.raises(ValueError):
        qo.layout(4, 8, 0, 5, 128)


# ---- the paper's own counts ---------------------------------------------------------
def _model_sum(golden, name, k, field):
    m = golden["models"][name]
    tot = 0
    for oc, ic in m["linears"]:
        lay = qo.layout(oc, ic, k, 4, 128)
        # information content of the group parameters: one fp16 scale + one fp16 zero-point per
        # group (the 16-byte row padding of the stored arrays is an alignment detail)
        tot += lay[field] if field != "group_bytes" else 4 * oc * lay["n_groups"]
    return tot * m["blocks"]


@pytest.mark.parametrize("name", ["7B", "13B", "70B"])
@pytest.mark.parametrize("k", [16, 128])
def test_tunable_parameter_counts_match_tab2(golden, name, k):
    """The FP16 weak block is OC x k in every linear layer: its element count over the
    whole model is the 'Tunable Params.' column of Tab. 2."""
    params = _model_sum(golden, name, k, "weak_bytes") // 2
    printed = golden["tunable_params_millions"][name][str(k)]
    assert round(params / 1e6) == printed


@pytest.mark.parametrize("name", ["7B", "13B", "70B"])
def test_group_parameter_storage_matches_tab8(golden, name):
    """Tab. 8: QEFT's storage exceeds OWQ's by the group-wise parameters.  OWQ keeps one
    (scale, zero) pair per output channel, QEFT one fp16 pair per group of 128, so
    QEFT - OWQ = 4 B * (#groups - #rows).  A different scale/zero width (2 B or 8 B per
    group) would miss the printed difference by a factor of two."""
    m = golden["models"][name]
    group_bytes = _model_sum(golden, name, 128, "group_bytes")
    rows = sum(oc for oc, _ in m["linears"]) * m["blocks"]
    delta_mib = (group_bytes - 4 * rows) / 2**20
    printed = golden["storage_mib_k128_4bit"][name]
    assert abs(delta_mib - (printed["qeft"] - printed["owq"])) / (printed["qeft"] - printed["owq"]) < 0.025


def test_weak_grad_cost_ratio_is_k_over_ic():
    """Sec. 3.3: flops of the weight gradient and the saved activation shrink to k/IC."""
    m, oc, ic, k = 4096, 11008, 4096, 128
    full = 2 * m * oc * ic
    weak = 2 * m * oc * k
    assert weak * ic == full * k
    assert (m * k) * ic == (m * ic) * k
