"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs.

Bit-exact for packing and quantizer decisions; relative error <= 2e-3 for outputs and
gradients (see parity_util.assert_close).  Sizes here are ones the oracle finishes in
seconds and that still span several tiles and ragged tails; the full benchmark shapes
are covered by test_gpu_fullsize.py on sampled outputs.
"""
import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth
from parity_util import HostLayer, assert_close, pad_cols

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------------------ packing
PACK_SHAPES = [  # oc, ic, k, bits, g
    (512, 512, 8, 4, 128),        # config 1: partial last group (Kq = 504)
    (96, 1024 + 128, 128, 4, 128),
    (80, 1280 + 128, 128, 3, 128),  # 3-bit: groups straddle words
    (33, 200, 24, 3, 64),
    (33, 200, 24, 4, 32),
    (17, 64, 64, 4, 128),         # every column weak
    (17, 72, 0, 3, 128),          # no weak column, single partial group
]


@pytest.mark.parametrize("oc,ic,k,bits,g", PACK_SHAPES)
def test_pack_rtn_bit_exact(oc, ic, k, bits, g):
    w = synth.make_weight(oc, ic, seed=oc + ic)
    if oc > 20:
        w[3, :min(g, ic - k)] = 0            # an all-zero group
        w[5, :] = np.abs(w[5, :])           # all-positive row: zero-point 0
        w[6, :] = -np.abs(w[6, :])          # all-negative row: zero-point qmax
    codes, scales, zeros, weak = qo.quantize_rtn(w, k, bits, g)
    lay = qo.layout(oc, ic, k, bits, g)
    ref_words = qo.pack_codes(codes, bits, lay["row_stride_words"])
    desc = B.make_desc(oc, ic, k, bits, g)
    _, wbuf = pad_cols(w)
    out = B.Weight(desc)
    out.qweight.fill_(-1)                    # the call must overwrite padding too
    B.qeft_pack(desc, wbuf[:, :ic], out)
    torch.cuda.synchronize()
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), ref_words)
    ng = lay["n_groups"]
    out.scales[:, ng:].fill_(1.0)            # padding must be rewritten as zero as well
    B.qeft_pack(desc, wbuf[:, :ic], out)
    torch.cuda.synchronize()
    assert out.scales.shape[1] == lay["group_stride"]
    assert np.array_equal(out.scales[:, :ng].cpu().numpy().view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(out.zeros[:, :ng].cpu().numpy().view(np.uint16), zeros.view(np.uint16))
    assert torch.all(out.scales[:, ng:] == 0) and torch.all(out.zeros[:, ng:] == 0)
    assert np.array_equal(out.weak.cpu().numpy().view(np.uint16), weak.view(np.uint16))


SEARCH_SHAPES = [  # oc, ic, k, bits, g, n_grid, step
    (512, 512, 8, 4, 128, 80, 0.01),          # config 1: partial last group
    (96, 1024 + 128, 128, 4, 128, 40, 0.02),
    (80, 1280 + 128, 128, 3, 128, 80, 0.01),  # 3-bit
    (40, 200, 40, 4, 32, 25, 0.03125),        # narrow groups: most lanes of a group idle
    (24, 136, 0, 3, 64, 1, 0.01),             # one candidate: plain min-max
]


@pytest.mark.parametrize("oc,ic,k,bits,g,n_grid,step", SEARCH_SHAPES)
def test_pack_search_bit_exact(oc, ic, k, bits, g, n_grid, step):
    """Grid-search quantizer (Sec. 3.1): on these seeded inputs no two candidates of a group are closer than the rounding
    of the kernel's fp32 error sum, so its choice equals the oracle's float64 first minimum and scales, zero-points and
    codes agree bit for bit (a regression pin; the criterion itself is checked order-free in the next test)."""
    w = synth.make_weight(oc, ic, seed=3 * oc + ic)
    w[1, 3] = np.float16(0.3)                # outliers, where truncation changes the choice
    w[2, min(g + 1, ic - k - 1)] = np.float16(-0.45)
    w[3, :min(g, ic - k)] = 0                # an all-zero group
    codes, scales, zeros, weak = qo.quantize_search(w, k, bits, g, n_grid, step)
    lay = qo.layout(oc, ic, k, bits, g)
    ref_words = qo.pack_codes(codes, bits, lay["row_stride_words"])
    desc = B.make_desc(oc, ic, k, bits, g)
    _, wbuf = pad_cols(w)
    out = B.Weight(desc)
    out.qweight.fill_(-1)
    out.scales.fill_(1.0)
    B.qeft_pack_search(desc, wbuf[:, :ic], n_grid, step, out)
    torch.cuda.synchronize()
    ng = lay["n_groups"]
    assert np.array_equal(out.scales[:, :ng].cpu().numpy().view(np.uint16), scales.view(np.uint16))
    assert np.array_equal(out.zeros[:, :ng].cpu().numpy().view(np.uint16), zeros.view(np.uint16))
    assert torch.all(out.scales[:, ng:] == 0) and torch.all(out.zeros[:, ng:] == 0)
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), ref_words)
    assert np.array_equal(out.weak.cpu().numpy().view(np.uint16), weak.view(np.uint16))
    if n_grid > 1:   # the search moved at least the outlier groups away from min-max
        _, s_rtn, _, _ = qo.quantize_rtn(w, k, bits, g)
        assert np.any(scales.view(np.uint16) != s_rtn.view(np.uint16))


@pytest.mark.parametrize("oc,ic,k,bits,g,n_grid,step", SEARCH_SHAPES + [(1024, 1024 + 128, 128, 4, 128, 80, 0.01), (300, 640, 0, 3, 64, 50, 0.015)])
def test_pack_search_reaches_the_minimum_whatever_the_summation_order(oc, ic, k, bits, g, n_grid, step):
    """The search is defined by its criterion (Sec. 3.1: the smallest squared weight error over the grid), not by an
    order of summation.  For every (row, group) the parameters the GPU chose must be one of the grid's candidates, its
    codes must be the round-to-nearest codes under those parameters, and the float64 error it reaches must not exceed
    the float64 minimum over the grid by more than 1e-5 relative (candidates closer than that are ties within the
    rounding of an fp32 error sum of up to 128 terms: 128 x 2^-24 = 7.6e-6)."""
    w = synth.make_weight(oc, ic, seed=5 * oc + ic)
    w[1, 3] = np.float16(0.3)
    w[3, :min(g, ic - k)] = 0
    desc = B.make_desc(oc, ic, k, bits, g)
    _, wbuf = pad_cols(w)
    out = B.Weight(desc)
    B.qeft_pack_search(desc, wbuf[:, :ic], n_grid, step, out)
    torch.cuda.synchronize()
    lay = qo.layout(oc, ic, k, bits, g)
    ng, kq = lay["n_groups"], lay["kq"]
    s_gpu = out.scales[:, :ng].cpu().numpy()
    z_gpu = out.zeros[:, :ng].cpu().numpy()
    codes_gpu = qo.unpack_codes(out.qweight.cpu().numpy().view(np.uint32), kq, bits)
    s_all, z_all, e_all = qo.search_candidates(w, k, bits, g, n_grid, step)
    is_cand = np.any((s_all.view(np.uint16) == s_gpu.view(np.uint16)[None]) & (z_all == z_gpu.astype(np.float32)[None]), axis=0)
    assert np.all(is_cand), "parameters that no candidate of the grid produces"
    assert np.array_equal(codes_gpu, qo.codes_for_params(w, k, bits, g, s_gpu, z_gpu))
    wq = qo.dequantize(codes_gpu, s_gpu, z_gpu, np.zeros((oc, 0), dtype=np.float16), g)
    d = (w[:, :kq].astype(np.float64) - wq) ** 2
    e_gpu = np.stack([d[:, gi * g:min((gi + 1) * g, kq)].sum(axis=1) for gi in range(ng)], axis=1)
    e_min = e_all.min(axis=0)
    assert np.all(e_gpu <= e_min * (1 + 1e-5) + 1e-30), f"worst excess {np.max(e_gpu / np.maximum(e_min, 1e-300)) - 1:.2e}"


@pytest.mark.parametrize("oc,ic,k,bits,g", PACK_SHAPES)
def test_pack_codes_and_unpack_bit_exact(oc, ic, k, bits, g):
    h = HostLayer(oc, ic, k, bits, g, seed=7 + oc)
    desc = h.desc
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    out = B.Weight(desc)
    out.qweight.fill_(-1)
    B.qeft_pack_codes(desc, dev(h.codes) if h.kq else None, dev(h.scales) if h.kq else None,
                      dev(h.zeros) if h.kq else None, dev(h.weak) if k else None, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), h.qweight)
    ng = h.lay["n_groups"]
    if h.kq:
        assert np.array_equal(out.scales[:, :ng].cpu().numpy().view(np.uint16), h.scales.view(np.uint16))
        assert np.array_equal(out.zeros[:, :ng].cpu().numpy().view(np.uint16), h.zeros.view(np.uint16))
        assert torch.all(out.scales[:, ng:] == 0) and torch.all(out.zeros[:, ng:] == 0)
    codes, scales, zeros, weak = B.qeft_unpack(desc, h.to_device())
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), h.codes)
    assert np.array_equal(scales.cpu().numpy().view(np.uint16), h.scales.view(np.uint16))
    assert np.array_equal(zeros.cpu().numpy().view(np.uint16), h.zeros.view(np.uint16))
    assert np.array_equal(weak.cpu().numpy().view(np.uint16), h.weak.view(np.uint16))


# ------------------------------------------------------------------------------ forward
FWD_CASES = [  # oc, ic, k, bits, g, Ms
    (512, 512, 8, 4, 128, [1, 16]),                  # config 1
    (528, 1024 + 128, 128, 4, 128, [1, 2, 3, 8, 13, 16, 17, 40]),   # ragged OC tile (528 = 33*16)
    (1000, 2048 + 64, 64, 4, 128, [1, 5]),           # OC not a multiple of 16
    (640, 1280 + 128, 128, 3, 128, [1, 4, 16]),      # 3-bit
    (512, 13696 % 1280 + 1280 + 128, 128, 3, 128, [1, 7]),   # 3-bit, row tail not a multiple of 40 codes
    (64, 333, 21, 4, 128, [1, 3]),                   # odd everything: generic path
    (64, 333, 21, 3, 32, [2]),
    (48, 256, 256, 4, 128, [1, 9, 40]),              # k = IC: plain fp16 layer (M = 40: the GEMM's direct fp16 stages alone)
    (200, 320, 320, 4, 128, [270]),                  # k = IC, odd number of stages, ragged OC and M
    (48, 384, 0, 4, 128, [1, 9]),                    # k = 0: pure group quantization
    (256, 1024 + 128, 128, 4, 128, [64, 300]),       # larger M: GEMM path, ragged M
    (384, 512 + 72, 72, 4, 128, [130]),              # k not a multiple of 32
    (272, 320 + 128, 128, 4, 128, [64, 257]),        # GEMM path, odd number of 64-column stages, ragged OC
    (256, 2560 + 256, 256, 4, 128, [33]),            # GEMM path, 20 groups (three reloads of the group parameters)
    (2064, 2176 + 64, 64, 4, 128, [5, 16]),          # unstaged decode kernel with a K split, 17 groups
    (2064, 2000 + 64, 64, 3, 128, [1, 6, 16]),       # 3-bit decode kernel with a K split, ragged OC
    (304, 4600 + 40, 40, 4, 128, [1, 7, 16]),        # 36 groups (the last partial): two passes of the register kernel, the second short
    (96, 10880 + 128, 128, 4, 128, [1, 6]),          # the 7B down projection's row length: three passes of eight waves
    (4112, 1024 + 256, 256, 4, 128, [1, 9]),         # 257 tiles, two waves per workgroup; weak block as wide as the register kernel takes
    (64, 512 + 288, 288, 4, 128, [1, 5]),            # weak block too wide for the register kernel: the unstaged kernel
    (8208, 4224 + 128, 128, 4, 128, [6, 16]),        # register kernel: 513 tiles with two passes over K - several tiles per workgroup, each in two passes
    (136, 17408 + 24, 24, 4, 128, [1, 3]),           # rows of 9 ranges of 2048 columns: the rows-per-wave kernel with two waves per row
    (360, 23552 + 16, 16, 4, 128, [1, 2]),           # 12 ranges: two waves of six
    (72, 26624 + 64, 64, 4, 128, [1, 5]),            # 13 ranges: four waves of four (three clamped)
]


@pytest.mark.parametrize("oc,ic,k,bits,g,Ms", FWD_CASES)
def test_forward_parity(oc, ic, k, bits, g, Ms):
    h = HostLayer(oc, ic, k, bits, g, seed=oc * 3 + ic)
    w = h.to_device()
    for m in Ms:
        x = synth.make_activations(m, ic, k, seed=m)
        xv, _ = pad_cols(x)
        y = B.qeft_linear_fwd(h.desc, w, xv)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"fwd {oc}x{ic} k{k} b{bits} M{m}")


def test_forward_rtn_quantized_layer_end_to_end():
    """qeft_pack on the GPU followed by qeft_linear_fwd equals the oracle's quantize -> dequantize -> matmul."""
    oc, ic, k, g, m = 512, 512, 8, 128, 16
    w16 = synth.make_weight(oc, ic, synth.seed_for(1, 0))
    x = synth.make_activations(m, ic, k, synth.seed_for(1, 0))
    desc = B.make_desc(oc, ic, k, 4, g)
    wd = B.qeft_pack(desc, torch.from_numpy(w16).cuda())
    y = B.qeft_linear_fwd(desc, wd, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    codes, scales, zeros, weak = qo.quantize_rtn(w16, k, 4, g)
    assert_close(y.cpu().numpy(), qo.linear_fwd(qo.dequantize(codes, scales, zeros, weak, g), x), "rtn end to end")


@pytest.mark.parametrize("m", [1, 16, 200])
def test_forward_exact_integer_case_is_bitwise(m):
    """Scales in {1, 0.5}, integer zero-points, small integer X and weak block: every partial
    sum is exact in fp32 whatever the reduction order, so the result must equal the oracle's
    fp16 rounding bit for bit."""
    r = np.random.default_rng(21)
    oc, kq, k, g = 272, 1024, 32, 128
    h = HostLayer(oc, kq + k, k, 4, g, seed=1)
    h.codes = r.integers(0, 16, size=(oc, kq), dtype=np.uint8)
    h.scales = r.choice([1.0, 0.5], size=(oc, kq // g)).astype(np.float16)
    h.zeros = r.integers(0, 16, size=(oc, kq // g)).astype(np.float16)
    h.weak = r.integers(-3, 4, size=(oc, k)).astype(np.float16)
    h.qweight = qo.pack_codes(h.codes, 4, h.lay["row_stride_words"])
    x = r.integers(-2, 3, size=(m, kq + k)).astype(np.float16)
    y = B.qeft_linear_fwd(h.desc, h.to_device(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    ref = qo.round_fp16(qo.linear_fwd(h.w64, x))
    assert np.array_equal(y.cpu().numpy().view(np.uint16), ref.view(np.uint16))


def test_forward_non_integer_zero_points():
    h = HostLayer(256, 512 + 32, 32, 4, 128, seed=5)
    h.zeros = np.random.default_rng(3).uniform(0, 15, size=h.zeros.shape).astype(np.float16)
    x = synth.make_activations(4, h.ic, h.k, 5)
    y = B.qeft_linear_fwd(h.desc, h.to_device(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), "float zero-points")


@pytest.mark.parametrize("m", [40, 300])
def test_gemm_paths_with_non_integer_zero_points(m):
    """The tiled kernels may not assume integer zero-points either (forward and input gradient)."""
    h = HostLayer(256, 512 + 128, 128, 4, 128, seed=11)
    h.zeros = np.random.default_rng(4).uniform(0, 15, size=h.zeros.shape).astype(np.float16)
    w = h.to_device()
    x = synth.make_activations(m, h.ic, h.k, 6)
    dy = synth.make_grad_output(m, h.oc, 7)
    y = B.qeft_linear_fwd(h.desc, w, torch.from_numpy(x).cuda())
    dx = B.qeft_linear_bwd_dx(h.desc, w, torch.from_numpy(dy).cuda())
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), "fwd, float zero-points")
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), "dX, float zero-points")


GROUP_CASES = [  # ic, k, bits, [oc per layer], Ms
    (1024 + 128, 128, 4, [256, 64, 64], [1, 3]),        # query / key / value of different widths
    (512 + 64, 64, 4, [176, 176], [1, 4]),              # gate / up; a workgroup straddles the two layers
    (2048 + 128, 128, 4, [40, 24, 520, 8], [2]),        # four layers, ragged tiles
    (1024 + 128, 128, 4, [256, 64], [9, 40]),           # more rows than the one-launch kernel takes: per-layer calls
    (640 + 40, 40, 3, [96, 32], [1]),                   # 3-bit: per-layer calls
]


@pytest.mark.parametrize("ic,k,bits,ocs,Ms", GROUP_CASES)
def test_forward_group_parity(ic, k, bits, ocs, Ms):
    """Layers that share an input, through qeft_linear_fwd_group: each output equals the oracle's."""
    hs = [HostLayer(oc, ic, k, bits, 128, seed=20 + i + oc) for i, oc in enumerate(ocs)]
    ws = [h.to_device() for h in hs]
    for m in Ms:
        x = synth.make_activations(m, ic, k, 31 + m)
        ys = B.qeft_linear_fwd_group([h.desc for h in hs], ws, torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        for i, (h, y) in enumerate(zip(hs, ys)):
            assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"group layer {i} (OC {h.oc}) M={m}")


@pytest.mark.parametrize("m", [1, 3, 8])
def test_forward_group_writes_only_its_outputs_and_repeats_bitwise(m):
    ic, k = 1024 + 128, 128
    hs = [HostLayer(oc, ic, k, 4, 128, seed=40 + oc) for oc in (200, 72)]
    ws = [h.to_device() for h in hs]
    x = torch.from_numpy(synth.make_activations(m, ic, k, 5)).cuda()
    bufs = [torch.full((m, h.oc + 16), -3.0, dtype=torch.float16, device="cuda") for h in hs]
    grp = B.Group([h.desc for h in hs], ws, [b[:, :h.oc] for b, h in zip(bufs, hs)])
    B.qeft_linear_fwd_group(None, None, x, group=grp)
    torch.cuda.synchronize()
    first = [b.clone() for b in bufs]
    for b, h in zip(bufs, hs):
        assert torch.all(b[:, h.oc:] == -3.0)              # nothing written past a layer's OC
        assert_close(b[:, :h.oc].cpu().numpy(), qo.linear_fwd(h.w64, x.cpu().numpy()), "group output")
    for _ in range(3):
        for b in bufs:
            b.fill_(-3.0)
        B.qeft_linear_fwd_group(None, None, x, group=grp)
        for b, f in zip(bufs, first):
            assert torch.equal(b, f)


@pytest.mark.parametrize("bits,dense", [(4, False), (3, False), (3, True)])
@pytest.mark.parametrize("m", [1, 2, 4, 6, 16, 40])
def test_forward_respects_leading_dimensions_and_is_deterministic(m, bits, dense):
    """Every forward kernel (one row, two to four, five to sixteen, the GEMM; 4-bit and both 3-bit layouts) on operands
    with leading dimensions larger than their widths: right values, nothing written past OC, bitwise repeatable."""
    h = HostLayer(320, 640 + 128, 128, bits, 128, seed=9, dense=dense)
    w = h.to_device()
    x = synth.make_activations(m, h.ic, h.k, 9)
    xbuf = torch.full((m, h.ic + 24), 7.0, dtype=torch.float16, device="cuda")
    xbuf[:, :h.ic].copy_(torch.from_numpy(x))
    ybuf = torch.full((m, h.oc + 8), -5.0, dtype=torch.float16, device="cuda")
    B.qeft_linear_fwd(h.desc, w, xbuf[:, :h.ic], ybuf[:, :h.oc])
    torch.cuda.synchronize()
    assert_close(ybuf[:, :h.oc].cpu().numpy(), qo.linear_fwd(h.w64, x), "strided fwd")
    assert torch.all(ybuf[:, h.oc:] == -5.0)              # nothing written past OC
    first = ybuf.clone()
    for _ in range(5):
        ybuf.fill_(-5.0)
        B.qeft_linear_fwd(h.desc, w, xbuf[:, :h.ic], ybuf[:, :h.oc])
        assert torch.equal(ybuf, first)                   # run-to-run bitwise equal (no atomics)


# ------------------------------------------------------------------------------ weak columns in place
IRREGULAR_CASES = [  # oc, ic, k, bits, Ms
    (256, 1024 + 128, 128, 4, [1, 3, 4, 5, 40]),   # gather inside the decode kernel (M <= 4), then behind a gather pass
    (4096, 4096, 128, 4, [1]),                  # the 7B output projection at full size
    (528, 2048 + 64, 64, 4, [2]),               # ragged last tile, weak block of two steps
    (272, 640 + 64, 64, 4, [300]),
    (96, 640 + 40, 40, 3, [1, 33]),            # 3-bit
    (64, 333, 21, 4, [5]),                     # odd sizes: generic kernels, ragged last chunk of the table
    (64, 384, 0, 4, [2]),                      # no weak column: the table is the identity
]


@pytest.mark.parametrize("oc,ic,k,bits,Ms", IRREGULAR_CASES)
def test_irregular_indices_parity(oc, ic, k, bits, Ms):
    """Weak columns at arbitrary channels (the un-reordered attention output projection): forward and
    input gradient against the oracle's gather / scatter definition."""
    h = HostLayer(oc, ic, k, bits, 128, seed=60 + oc)
    w = h.to_device()
    r = np.random.default_rng(ic)
    weak_idx = r.permutation(ic)[:k]           # arbitrary places, arbitrary order
    perm = qo.stored_order(ic, weak_idx)
    perm_d = torch.from_numpy(perm).cuda()
    for m in Ms:
        x = synth.make_activations(m, ic, 0, 70 + m)
        x[:, weak_idx] *= 20.0                 # the outlier channels sit where the weak columns are
        dy = synth.make_grad_output(m, oc, 71 + m)
        _, xbuf = pad_cols(x)                  # leading dimension a multiple of 8
        y = B.qeft_linear_fwd_irregular(h.desc, w, perm_d, xbuf[:, :ic])
        dx = B.qeft_linear_bwd_dx_irregular(h.desc, w, perm_d, torch.from_numpy(dy).cuda())
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), qo.linear_fwd_irregular(h.w64, perm, x), f"irregular fwd M={m}")
        assert_close(dx.cpu().numpy(), qo.linear_bwd_dx_irregular(h.w64, perm, dy), f"irregular dX M={m}")


def test_irregular_malformed_table_stays_in_bounds():
    """Entries outside 0 .. IC-1 are clamped: wrong numbers, but nothing outside X / dX is touched."""
    h = HostLayer(64, 256 + 128, 128, 4, 128, seed=3)
    w = h.to_device()
    ic, m = h.ic, 4
    perm = torch.full((ic,), 10 ** 6, dtype=torch.int32, device="cuda")
    perm[::2] = -7
    xbuf = torch.zeros((m + 2, ic), dtype=torch.float16, device="cuda")
    xbuf[0].fill_(float("nan")); xbuf[-1].fill_(float("nan"))      # guard rows around X
    xbuf[1:-1] = 1.0
    y = B.qeft_linear_fwd_irregular(h.desc, w, perm, xbuf[1:-1])
    dbuf = torch.full((m + 2, ic), 5.0, dtype=torch.float16, device="cuda")
    B.qeft_linear_bwd_dx_irregular(h.desc, w, perm, torch.ones((m, h.oc), dtype=torch.float16, device="cuda"), dbuf[1:-1])
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(y))                             # no guard row was read
    assert torch.all(dbuf[0] == 5.0) and torch.all(dbuf[-1] == 5.0)  # no guard row was written


# ------------------------------------------------------------------------------ global weak columns, reordering
@pytest.mark.parametrize("tokens,d,n_batch", [(64, 96, 4), (700, 4096, 7), (33, 1032, 3)])
def test_sensitivity_parity(tokens, d, n_batch):
    x = synth.make_activations(tokens, d, 16, tokens + d)
    got = B.qeft_sensitivity(pad_cols(x)[0], n_batch).cpu().numpy().astype(np.float64)
    ref = qo.sensitivity(x, n_batch)
    np.testing.assert_allclose(got, ref, rtol=2e-6)            # fp32 sums of fp32 squares


def test_global_weak_columns_end_to_end():
    """Planted outlier channels (Sec. 3.2): sensitivity, per-layer votes, global top-k, the reordering
    permutation and the reordered matrices all equal the oracle's; the reordered layer's output does not change."""
    r = np.random.default_rng(8)
    d, k, oc, planted = 1024, 16, 128, sorted(r.permutation(1024)[:16].tolist())
    layers = []
    for li in range(4):
        x = r.standard_normal((96, d)).astype(np.float32) * (1.0 + li)      # layers of different overall scale
        x[:, planted] *= 15.0
        if li == 1:
            x[:, (planted[0] + 1) % d] *= 20.0                               # an outlier only this layer has: one vote, not four
        layers.append(x.astype(np.float16))
    s_global = torch.zeros(d, dtype=torch.float32, device="cuda")
    ref_global = np.zeros(d)
    for x in layers:
        s_local = B.qeft_sensitivity(torch.from_numpy(x).cuda(), 4)
        ids = B.qeft_vote(s_local, k, s_global)
        ref_ids = qo.vote(qo.sensitivity(x, 4), k, ref_global)
        assert sorted(ids.cpu().tolist()) == sorted(ref_ids.tolist())        # clear margins: the same channels
    np.testing.assert_allclose(s_global.cpu().numpy(), ref_global, rtol=1e-5)
    idx = B.qeft_vote(s_global, k)
    ref_idx = qo.global_weak_columns([(x, 4) for x in layers], k)
    assert sorted(idx.cpu().tolist()) == planted == sorted(ref_idx.tolist())
    perm = B.qeft_weak_order(idx, d)
    assert np.array_equal(perm.cpu().numpy(), qo.stored_order(d, idx.cpu().numpy()))
    # reorder a weight along its columns and the activations with it; along its rows for a producer
    w = synth.make_weight(oc, d, seed=5)
    wr = B.qeft_reorder(torch.from_numpy(w).cuda(), perm, 1)
    xr = B.qeft_reorder(torch.from_numpy(layers[0]).cuda(), perm, 1)
    p = perm.cpu().numpy()
    assert np.array_equal(wr.cpu().numpy().view(np.uint16), qo.reorder(w, p, 1).view(np.uint16))
    assert np.array_equal(xr.cpu().numpy().view(np.uint16), qo.reorder(layers[0], p, 1).view(np.uint16))
    v = synth.make_weight(d, 256, seed=6)
    vr = B.qeft_reorder(torch.from_numpy(v).cuda(), perm, 0)
    assert np.array_equal(vr.cpu().numpy().view(np.uint16), qo.reorder(v, p, 0).view(np.uint16))
    # the reordered layer, quantized with its weak columns now last, reproduces the original product
    desc = B.make_desc(oc, d, k, 4, 128)
    y = B.qeft_linear_fwd(desc, B.qeft_pack(desc, wr), xr[:8])
    wq = qo.quantize_rtn(qo.reorder(w, p, 1), k, 4, 128)
    w64 = qo.dequantize(*wq, 128)
    assert_close(y.cpu().numpy(), qo.linear_fwd(w64, qo.reorder(layers[0][:8], p, 1)), "reordered layer")
    dense = layers[0][:8].astype(np.float64) @ w.astype(np.float64).T        # the un-reordered fp16 layer
    rel = np.linalg.norm(y.cpu().numpy() - dense) / np.linalg.norm(dense)
    assert rel < 0.05                                                        # quantization error only


def test_vote_ties_and_plain_top_k():
    v = torch.tensor([1.0, 5.0, 3.0, 5.0, 0.0, 3.0], device="cuda")
    assert B.qeft_vote(v, 4).cpu().tolist() == qo.top_k(v.cpu().numpy(), 4).tolist() == [1, 3, 2, 5]
    sg = torch.zeros(6, device="cuda")
    B.qeft_vote(v, 2, sg)
    ref = np.zeros(6)
    qo.vote(v.cpu().numpy(), 2, ref)
    np.testing.assert_allclose(sg.cpu().numpy(), ref, rtol=1e-6)


def test_merge_weak_bit_exact():
    """QEFT merging (Sec. 5): into the columns of a full-precision target and into a weak block."""
    r = np.random.default_rng(12)
    oc, ic, k = 300, 520, 40
    t = r.standard_normal((oc, ic)).astype(np.float16)
    a0 = (r.standard_normal((oc, k)) * 0.02).astype(np.float16)
    a1 = (a0.astype(np.float32) + r.standard_normal((oc, k)).astype(np.float32) * 0.003).astype(np.float16)
    idx = r.permutation(ic)[:k].astype(np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    full = B.qeft_merge_weak(dev(a1), dev(a0), dev(t), dev(idx))
    blk = B.qeft_merge_weak(dev(a1), dev(a0), dev(t[:, idx]))
    torch.cuda.synchronize()
    assert np.array_equal(full.cpu().numpy().view(np.uint16), qo.merge_weak(t, a1, a0, idx).view(np.uint16))
    assert np.array_equal(blk.cpu().numpy().view(np.uint16), qo.merge_weak(t[:, idx], a1, a0).view(np.uint16))


# ------------------------------------------------------------------------------ backward
BWD_CASES = [  # oc, ic, k, bits, g, M
    (256, 512 + 128, 128, 4, 128, 300),
    (528, 1024 + 128, 128, 4, 128, 64),
    (200, 333, 21, 4, 128, 5),        # generic
    (200, 640 + 40, 40, 3, 128, 33),  # 3-bit backward
    (64, 256, 256, 4, 128, 17),       # k = IC
    (64, 384, 0, 4, 128, 17),         # k = 0
    (384, 512 + 72, 72, 4, 128, 130),
    (128, 384 + 128, 128, 4, 128, 70),   # a tile whose first half is quantized and second half weak
    (64, 128 + 256, 256, 4, 128, 290),   # mixed tile, then an all-weak tile with a dead half
    (192, 256 + 40, 40, 4, 128, 40),     # weak half narrower than 128 channels
    (320, 896, 0, 4, 128, 257),          # no weak block, last tile half empty, odd stage count
]


@pytest.mark.parametrize("oc,ic,k,bits,g,m", BWD_CASES)
def test_backward_dx_parity(oc, ic, k, bits, g, m):
    h = HostLayer(oc, ic, k, bits, g, seed=oc + 5 * ic)
    dy = synth.make_grad_output(m, oc, seed=m)
    dyv, _ = pad_cols(dy)
    dx = B.qeft_linear_bwd_dx(h.desc, h.to_device(), dyv)
    torch.cuda.synchronize()
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"dX {oc}x{ic} k{k} b{bits} M{m}")


@pytest.mark.parametrize("oc,ic,k,bits,g,m", BWD_CASES)
@pytest.mark.parametrize("compact", [False, True])
def test_weak_grad_parity(oc, ic, k, bits, g, m, compact):
    if k == 0:
        pytest.skip("no weak block")
    desc = B.make_desc(oc, ic, k, bits, g)
    x = synth.make_activations(m, ic, k, seed=m + 1)
    dy = synth.make_grad_output(m, oc, seed=m + 2)
    dyv, _ = pad_cols(dy)
    kq = ic - k
    if compact or kq % 8:
        xw, _ = pad_cols(x[:, kq:])                      # the saved k-wide copy
    else:
        xv, _ = pad_cols(x)
        xw = xv[:, kq:]                                  # a view into the full activation
    ref = qo.weak_grad(dy, x[:, kq:])
    dw = B.qeft_weak_grad(desc, dyv, xw, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert_close(dw.cpu().numpy(), ref, f"dW {oc}x{k} M{m}")
    # accumulate: dW += grad, fp16 output
    base = (np.random.default_rng(1).standard_normal((oc, k)) * 0.05).astype(np.float16)
    dw16 = torch.from_numpy(base).cuda()
    B.qeft_weak_grad(desc, dyv, xw, dW=dw16, accumulate=True)
    torch.cuda.synchronize()
    assert_close(dw16.cpu().numpy(), base.astype(np.float64) + ref, f"dW accumulate {oc}x{k}")
    dw16.fill_(3.0)
    B.qeft_weak_grad(desc, dyv, xw, dW=dw16, accumulate=False)
    torch.cuda.synchronize()
    assert_close(dw16.cpu().numpy(), ref, f"dW overwrite {oc}x{k}")


@pytest.mark.parametrize("oc,ic,k,bits,g,m", BWD_CASES + [
    (704, 1024 + 128, 128, 4, 128, 600),      # 5 x 3 tiles and 11 strips x 8 token splits in one launch
    (2816, 512 + 256, 256, 4, 128, 1024),     # a weak block of two halves; more strips than tiles
    (1088, 8320 + 128, 128, 4, 128, 300),     # 33 x 2 tiles: the strips fill the second round
])
def test_backward_in_one_call_equals_the_two_calls(oc, ic, k, bits, g, m):
    """qeft_linear_bwd: dX and dW_weak of a layer in one call (one launch where both take the tensor-core path): bit for
    bit what qeft_linear_bwd_dx (no workspace) and qeft_weak_grad give, and the oracle's values to the bar."""
    h = HostLayer(oc, ic, k, bits, g, seed=oc + 7 * ic)
    w = h.to_device()
    x = synth.make_activations(m, ic, k, seed=m + 3)
    dy = synth.make_grad_output(m, oc, seed=m + 4)
    dyv, _ = pad_cols(dy)
    kq = ic - k
    xw = pad_cols(x[:, kq:])[0] if k else None
    for dtype, acc in ((torch.float32, False), (torch.float16, True)):
        base = (np.random.default_rng(2).standard_normal((oc, k)) * 0.05).astype(np.float16)
        dw_a = torch.from_numpy(base).cuda().to(dtype) if k else None
        dw_b = dw_a.clone() if k else None
        dx_a = B.qeft_linear_bwd_dx(h.desc, w, dyv, ws=False)
        if k:
            B.qeft_weak_grad(h.desc, dyv, xw, dW=dw_a, accumulate=acc)
        if k:
            dx_b, _ = B.qeft_linear_bwd(h.desc, w, dyv, xw, dW=dw_b, accumulate=acc)
        else:
            dx_b = torch.empty_like(dx_a)
            B._check(B.raw.qeft_linear_bwd(B.C.byref(h.desc), B.C.byref(w.c_struct()), dyv.data_ptr(), m, dyv.stride(0), dx_b.data_ptr(),
                                           dx_b.stride(0), None, 0, None, 1, 0, None, 0, None), "qeft_linear_bwd")
        torch.cuda.synchronize()
        assert torch.equal(dx_a, dx_b)
        if k:
            assert torch.equal(dw_a, dw_b)
    assert_close(dx_b.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"dX {oc}x{ic} (one call)")
    if k:
        assert_close(dw_b.float().cpu().numpy(), base.astype(np.float64) + qo.weak_grad(dy, x[:, kq:]), f"dW {oc}x{k} (one call)")


@pytest.mark.parametrize("oc,ic,k,m", [
    (2048, 1024 + 128, 128, 512),    # 5 x 2 tiles: every tile's rows split
    (4096, 5120, 128, 4096),         # 20 x 16 tiles: the 64 of the last round split four ways
])
def test_backward_in_one_call_with_room_for_a_row_split(oc, ic, k, m):
    """qeft_linear_bwd with a workspace of QEFT_OP_BWD's size: dX takes the row split, the weak gradient follows in the
    same bytes: bit for bit qeft_linear_bwd_dx with its workspace, then qeft_weak_grad."""
    h = HostLayer(oc, ic, k, 4, 128, seed=oc + ic)
    w = h.to_device()
    gen = torch.Generator(device="cuda").manual_seed(m)
    x = torch.randn((m, ic), generator=gen, device="cuda").half()
    dy = (torch.randn((m, oc), generator=gen, device="cuda") * 0.01).half()
    n_dx = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD_DX, m)
    n_dw = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_WEAK_GRAD, m)
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD, m)
    assert n_dx > 0 and n == max(n_dx, n_dw)
    ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    dx_a = B.qeft_linear_bwd_dx(h.desc, w, dy, ws=ws)
    dw_a = B.qeft_weak_grad(h.desc, dy, x[:, ic - k:], ws=ws)
    ws.fill_(0xFF)
    dx_b, dw_b = B.qeft_linear_bwd(h.desc, w, dy, x[:, ic - k:], ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(dx_a, dx_b) and torch.equal(dw_a, dw_b)
    # the split really ran (the unsplit kernel rounds once less), and it is the room that decides: with the weak
    # gradient's amount alone the call splits only where that amount happens to be enough
    dx_u = B.qeft_linear_bwd_dx(h.desc, w, dy, ws=False)
    assert not torch.equal(dx_u, dx_b)
    dx_c, _ = B.qeft_linear_bwd(h.desc, w, dy, x[:, ic - k:], ws=torch.empty(max(n_dw, 16), dtype=torch.uint8, device="cuda"))
    assert torch.equal(dx_c, dx_b if n_dw >= n_dx else dx_u)


@pytest.mark.parametrize("dense", [False, True])
def test_backward_in_one_call_three_bit(dense):
    """qeft_linear_bwd on a 3-bit layer: with a workspace of QEFT_OP_BWD's size dX runs the tensor-core kernels on the fp16
    copy (bit for bit qeft_linear_bwd_dx with that workspace, then qeft_weak_grad); with the weak gradient's amount alone
    it still gives the right values, through the general kernel."""
    oc, ic, k, m = 528, 1280 + 128, 128, 300
    h = HostLayer(oc, ic, k, 3, 128, seed=77, dense=dense)
    w = h.to_device()
    x = synth.make_activations(m, ic, k, seed=5)
    dy = synth.make_grad_output(m, oc, seed=6)
    dyt, xw = torch.from_numpy(dy).cuda(), torch.from_numpy(np.ascontiguousarray(x[:, ic - k:])).cuda()
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD, m)
    assert n >= oc * ic * 2
    ws = torch.empty(n, dtype=torch.uint8, device="cuda")
    dx_a = B.qeft_linear_bwd_dx(h.desc, w, dyt, ws=ws)
    dw_a = B.qeft_weak_grad(h.desc, dyt, xw, ws=ws)
    dx_b, dw_b = B.qeft_linear_bwd(h.desc, w, dyt, xw, ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(dx_a, dx_b) and torch.equal(dw_a, dw_b)
    dx_c, dw_c = B.qeft_linear_bwd(h.desc, w, dyt, xw)                       # the weak gradient's workspace only
    torch.cuda.synchronize()
    for dx, dw, what in ((dx_b, dw_b, "copy"), (dx_c, dw_c, "general")):
        assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"dX 3-bit one call ({what})")
        assert_close(dw.cpu().numpy(), qo.weak_grad(dy, x[:, ic - k:]), f"dW 3-bit one call ({what})")


@pytest.mark.parametrize("oc,ic,k,m", [
    (256, 4096 + 128, 128, 300),     # 2 tiles, 64 quantized stages: 8 splits of 8 stages, the weak block in the last
    (528, 2560 + 64, 64, 64),        # 3 tiles (one ragged), 40 stages: 5 splits
    (200, 1088 + 72, 72, 130),       # 17 stages: splits of 16 and 1 stage, ragged weak block (LDS-staged weak stages in the last split)
    (1000, 3072, 0, 100),            # no weak block
    (8448, 2048 + 128, 128, 2048),   # 264 tiles: 32 per XCD unsplit, the 33rd of each XCD in 4 splits
    (9448, 2048 + 128, 128, 1700),   # 259 tiles (ragged both ways): the last XCD has fewer tiles and no split one
])
def test_forward_k_split_with_workspace(oc, ic, k, m):
    """Forward launches of few tiles, or whose last round of tiles fills few CUs: with the optional workspace the K
    range of those tiles is split over workgroups and the fp16 partial tiles are summed by a second kernel; without it
    one workgroup per tile walks the whole range."""
    h = HostLayer(oc, ic, k, 4, 128, seed=oc + ic)
    w = h.to_device()
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_FWD, m)
    assert n > 0 and n % (256 * 256 * 2) == 0       # whole partial tiles
    x = synth.make_activations(m, ic, k, seed=m)
    xv, _ = pad_cols(x)
    ws = torch.full((n + 64,), 0x7f, dtype=torch.uint8, device="cuda")
    ybuf = torch.full((m, oc + 8), -5.0, dtype=torch.float16, device="cuda")
    ref = qo.linear_fwd(h.w64, x)
    for use_ws in (ws[:n], False):
        ybuf.fill_(-5.0)
        B.qeft_linear_fwd(h.desc, w, xv, ybuf[:, :oc], ws=use_ws)
        torch.cuda.synchronize()
        assert_close(ybuf[:, :oc].cpu().numpy(), ref, f"fwd {oc}x{ic} M{m} ws={use_ws is not False}")
        assert torch.all(ybuf[:, oc:] == -5.0)
    assert torch.all(ws[n:] == 0x7f)
    with pytest.raises(B.QeftError):
        B.qeft_linear_fwd(h.desc, w, xv, ws=ws[:n - 16])   # too small


@pytest.mark.parametrize("oc,ic,k,m", [
    (4096, 256 + 128, 128, 300),     # 2 x 2 tiles (the second half weak, then empty), 64 stages of rows: 8 splits
    (1088, 640, 0, 64),              # 17 stages: splits of 16 and 1, no weak block
    (2560, 1024 + 64, 64, 130),      # mixed last tile, 40 stages: 5 splits
    (2048, 8320 + 128, 128, 2048),   # 264 tiles: the 33rd of each XCD (the half-quantized, half-weak last one) in 4 splits
    (2112, 9344 + 128, 128, 1700),   # 259 tiles (split ones all quantized), 33 stages: 3 splits, the last of one stage
])
def test_backward_dx_row_split_with_workspace(oc, ic, k, m):
    """Input-gradient launches of few tiles, or whose last round fills few CUs: with the optional workspace the weight
    rows of those tiles are split over workgroups (fp16 partial tiles, summed by a second kernel); without it one
    workgroup per tile walks all rows."""
    h = HostLayer(oc, ic, k, 4, 128, seed=oc + ic)
    w = h.to_device()
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD_DX, m)
    assert n > 0 and n % (256 * 256 * 2) == 0       # whole partial tiles
    dy = synth.make_grad_output(m, oc, seed=m)
    dyv, _ = pad_cols(dy)
    ws = torch.full((n + 64,), 0x7f, dtype=torch.uint8, device="cuda")
    buf = torch.full((m, ic + 8), -5.0, dtype=torch.float16, device="cuda")
    ref = qo.linear_bwd_dx(h.w64, dy)
    for use_ws in (ws[:n], False):
        buf.fill_(-5.0)
        B.qeft_linear_bwd_dx(h.desc, w, dyv, buf[:, :ic], ws=use_ws)
        torch.cuda.synchronize()
        assert_close(buf[:, :ic].cpu().numpy(), ref, f"dX {oc}x{ic} M{m} ws={use_ws is not False}")
        assert torch.all(buf[:, ic:] == -5.0)
    assert torch.all(ws[n:] == 0x7f)
    with pytest.raises(B.QeftError):
        B.qeft_linear_bwd_dx(h.desc, w, dyv, ws=ws[:n - 16])   # too small


@pytest.mark.parametrize("dense", [False, True])
def test_three_bit_gemm_splits_the_copy(dense):
    """3-bit layers at GEMM sizes: behind the fp16 copy the workspace may hold the partial tiles of a split of the copy
    (few tiles here; forward: 18 stages of columns -> 3 splits, input gradient: 16 stages of rows -> 2 splits); with room
    for the copy only, one workgroup per tile."""
    oc, ic, k, m = 1024, 1024 + 128, 128, 300
    h = HostLayer(oc, ic, k, 3, 128, seed=5, dense=dense)
    w = h.to_device()
    copy = oc * ic * 2
    nf, nd = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_FWD, m), B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD_DX, m)
    for n in (nf, nd):
        assert n > copy and (n - copy) % (256 * 256 * 2) == 0
    x = synth.make_activations(m, ic, k, seed=m)
    xv, _ = pad_cols(x)
    dy = synth.make_grad_output(m, oc, seed=m)
    dyv, _ = pad_cols(dy)
    ref_y, ref_dx = qo.linear_fwd(h.w64, x), qo.linear_bwd_dx(h.w64, dy)
    n = max(nf, nd)
    ws = torch.full((n + 64,), 0x7f, dtype=torch.uint8, device="cuda")
    for use in (ws[:n], ws[:copy]):
        y = B.qeft_linear_fwd(h.desc, w, xv, ws=use)
        dx = B.qeft_linear_bwd_dx(h.desc, w, dyv, ws=use)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), ref_y, f"3-bit fwd {oc}x{ic} M{m}, workspace {use.numel()} bytes")
        assert_close(dx.cpu().numpy(), ref_dx, f"3-bit dX {oc}x{ic} M{m}, workspace {use.numel()} bytes")
    assert torch.all(ws[n:] == 0x7f)


@pytest.mark.parametrize("dense", [False, True])
@pytest.mark.parametrize("oc,ic,k,m", [(320, 1280 + 128, 128, 300), (264, 512 + 64, 64, 40)])
def test_three_bit_gemm_sizes_through_the_fp16_copy(oc, ic, k, m, dense):
    """3-bit layers at M > 16: dequantized once into the workspace, then the tensor-core kernels; the same
    results (to the bar) without a workspace, from the general kernel."""
    h = HostLayer(oc, ic, k, 3, 128, seed=oc + ic, dense=dense)
    w = h.to_device()
    nbytes = oc * ic * 2                                   # the copy; behind it, partial tiles when the GEMM on the copy is split
    n = max(B.qeft_workspace_bytes(h.desc, op, m) for op in (B.QEFT_OP_FWD, B.QEFT_OP_BWD_DX))
    for op in (B.QEFT_OP_FWD, B.QEFT_OP_BWD_DX):
        extra = B.qeft_workspace_bytes(h.desc, op, m) - nbytes
        assert extra >= 0 and extra % (256 * 256 * 2) == 0
    assert B.qeft_workspace_bytes(h.desc, B.QEFT_OP_FWD, 16) == 0
    x = synth.make_activations(m, ic, k, seed=m)
    dy = synth.make_grad_output(m, oc, seed=m)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    ws = torch.full((n + 64,), 0x7f, dtype=torch.uint8, device="cuda")
    for use_ws in (ws[:n], False):
        y = B.qeft_linear_fwd(h.desc, w, xd, ws=use_ws)
        dx = B.qeft_linear_bwd_dx(h.desc, w, dyd, ws=use_ws)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"3-bit fwd M{m} ws={use_ws is not False}")
        assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"3-bit dX M{m} ws={use_ws is not False}")
    assert torch.all(ws[n:] == 0x7f)                       # nothing written past the stated size
    # the copy is the dequantized layer, rounded once to fp16
    copy = ws[:nbytes].view(torch.float16).reshape(oc, ic).cpu().numpy()
    assert np.array_equal(copy, h.w64.astype(np.float32).astype(np.float16)) or \
        np.max(np.abs(copy.astype(np.float64) - h.w64)) <= np.max(np.abs(h.w64)) * 2.0 ** -11
    with pytest.raises(B.QeftError):
        B.qeft_linear_fwd(h.desc, w, xd, ws=ws[:nbytes - 16])   # too small for the copy
    # the weak block is trainable: a call after an update must not reuse the old copy
    new_weak = (np.random.default_rng(3).standard_normal((oc, k)) * 0.05).astype(np.float16)
    w.weak.copy_(torch.from_numpy(new_weak))
    w64 = qo.dequantize(h.codes, h.scales, h.zeros, new_weak, 128)
    y = B.qeft_linear_fwd(h.desc, w, xd, ws=ws[:n])
    dx = B.qeft_linear_bwd_dx(h.desc, w, dyd, ws=ws[:n])
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), qo.linear_fwd(w64, x), "3-bit fwd after a weak-block update")
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(w64, dy), "3-bit dX after a weak-block update")


def test_backward_uses_current_weak_values():
    """dX goes through whatever the weak block holds now (it is the trainable tensor)."""
    h = HostLayer(128, 256 + 64, 64, 4, 128, seed=2)
    w = h.to_device()
    dy = synth.make_grad_output(20, h.oc, 3)
    new_weak = (np.random.default_rng(4).standard_normal(h.weak.shape) * 0.1).astype(np.float16)
    w.weak.copy_(torch.from_numpy(new_weak))
    dx = B.qeft_linear_bwd_dx(h.desc, w, torch.from_numpy(dy).cuda())
    torch.cuda.synchronize()
    w64 = qo.dequantize(h.codes, h.scales, h.zeros, new_weak, h.g)
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(w64, dy), "dX after weak update")


def test_empty_batch_is_a_no_op():
    h = HostLayer(64, 256, 128, 4, 128, seed=2)
    w = h.to_device()
    x = torch.empty((0, 256), dtype=torch.float16, device="cuda")
    assert B.qeft_linear_fwd(h.desc, w, x).shape == (0, 64)
    dy = torch.empty((0, 64), dtype=torch.float16, device="cuda")
    assert B.qeft_linear_bwd_dx(h.desc, w, dy).shape == (0, 256)
    dw = torch.full((64, 128), 2.0, dtype=torch.float32, device="cuda")
    B.qeft_weak_grad(h.desc, dy, x[:, 128:], dW=dw)
    torch.cuda.synchronize()
    assert torch.all(dw == 2.0)


# ------------------------------------------------------------------------------ exact-arithmetic and repeat pins
def _integer_layer(oc, kq, k, seed):
    """A stored layer whose weights are small integers: scale 1, zero-point 7 or 8, so s (q - z) lies in -8 .. 8 and is
    exact in fp16; weak block integers in -3 .. 3.  With integer activations in -1 .. 1 every product and every partial
    sum of a few thousand terms is an integer below 2048: exact in fp32 in ANY order of summation and exact in fp16,
    also where a split launch stores fp16 partial tiles.  The GPU must then equal the oracle bit for bit."""
    r = np.random.default_rng(seed)
    h = HostLayer(oc, kq + k, k, 4, 128, seed=1)
    ng = h.lay["n_groups"]
    h.codes = r.integers(0, 16, size=(oc, kq), dtype=np.uint8)
    h.scales = np.ones((oc, ng), dtype=np.float16)
    h.zeros = r.integers(7, 9, size=(oc, ng)).astype(np.float16)
    h.weak = r.integers(-3, 4, size=(oc, k)).astype(np.float16)
    h.qweight = qo.pack_codes(h.codes, 4, h.lay["row_stride_words"])
    return h, r


def _bitwise(t, ref64, what):
    ref = qo.round_fp16(ref64)
    assert np.max(np.abs(ref64)) < 2048, "the case left the range in which every value is exact"
    assert np.array_equal(t.cpu().numpy().view(np.uint16), ref.view(np.uint16)), what


@pytest.mark.parametrize("oc,kq,k,m,split", [
    (272, 1024, 32, 200, False),      # one workgroup per tile
    (256, 4096, 128, 300, True),      # 2 tiles, K split 8 ways over the workspace
    (8448, 2048, 128, 512, True),     # 33 x 2 tiles: the last round's tiles split
])
def test_forward_gemm_exact_integer_case_is_bitwise(oc, kq, k, m, split):
    h, r = _integer_layer(oc, kq, k, seed=31)
    x = r.integers(-1, 2, size=(m, kq + k)).astype(np.float16)
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_FWD, m)
    assert n > 0 or not split
    ws = torch.empty(n, dtype=torch.uint8, device="cuda") if split else False
    y = B.qeft_linear_fwd(h.desc, h.to_device(), torch.from_numpy(x).cuda(), ws=ws)
    torch.cuda.synchronize()
    _bitwise(y, qo.linear_fwd(h.w64, x), f"fwd {oc}x{kq + k} M{m} split={split}")


@pytest.mark.parametrize("oc,kq,k,m,split", [
    (320, 768, 128, 257, False),      # mixed last tile, one workgroup per tile
    (4096, 256, 128, 300, True),      # 64 stages of rows: 8 splits
    (2048, 8320, 128, 512, True),     # 33 x 2 tiles: the last round's tiles split over the weight rows
])
def test_backward_dx_exact_integer_case_is_bitwise(oc, kq, k, m, split):
    h, r = _integer_layer(oc, kq, k, seed=32)
    dy = r.integers(-1, 2, size=(m, oc)).astype(np.float16)
    n = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD_DX, m)
    assert n > 0 or not split
    ws = torch.empty(n, dtype=torch.uint8, device="cuda") if split else False
    dx = B.qeft_linear_bwd_dx(h.desc, h.to_device(), torch.from_numpy(dy).cuda(), ws=ws)
    torch.cuda.synchronize()
    _bitwise(dx, qo.linear_bwd_dx(h.w64, dy), f"dX {oc}x{kq + k} M{m} split={split}")


@pytest.mark.parametrize("oc,k,m", [(256, 128, 4096), (704, 256, 1000), (64, 40, 64)])
def test_weak_grad_exact_integer_case_is_bitwise(oc, k, m):
    """Integer dY and weak activations in -2 .. 2: every partial sum (token splits, slab sums) is an exact integer, so
    the fp32 result equals the oracle's exactly and the fp16 one its rounding."""
    r = np.random.default_rng(33)
    desc = B.make_desc(oc, 512 + k, k, 4, 128)
    dy = r.integers(-2, 3, size=(m, oc)).astype(np.float16)
    xw = r.integers(-2, 3, size=(m, k)).astype(np.float16)
    ref = qo.weak_grad(dy, xw)
    dyd, xwd = torch.from_numpy(dy).cuda(), pad_cols(xw)[0]
    dw32 = B.qeft_weak_grad(desc, dyd, xwd, out_dtype=torch.float32)
    dw16 = B.qeft_weak_grad(desc, dyd, xwd, out_dtype=torch.float16)
    torch.cuda.synchronize()
    assert np.array_equal(dw32.cpu().numpy().astype(np.float64), ref)
    assert np.array_equal(dw16.cpu().numpy().view(np.uint16), qo.round_fp16(ref).view(np.uint16))


@pytest.mark.parametrize("oc,ic,k,m,use_ws", [
    (320, 768 + 128, 128, 257, False),
    (4096, 256 + 128, 128, 300, True),       # row split of dX / its forward takes one tile row
    (256, 4096 + 128, 128, 300, True),       # K split of the forward
    (2048, 2048 + 128, 128, 2300, True),     # 9 x 9 tiles
])
def test_gemm_paths_repeat_bitwise(oc, ic, k, m, use_ws):
    """No atomics anywhere: forward, input gradient (split or not) and the two-pass weak gradient give the same bits
    on every run."""
    h = HostLayer(oc, ic, k, 4, 128, seed=oc + ic)
    w = h.to_device()
    xd = torch.from_numpy(synth.make_activations(m, ic, k, 3)).cuda()
    dyd = torch.from_numpy(synth.make_grad_output(m, oc, 4)).cuda()
    nf, nd = B.qeft_workspace_bytes(h.desc, B.QEFT_OP_FWD, m), B.qeft_workspace_bytes(h.desc, B.QEFT_OP_BWD_DX, m)
    wsf = torch.empty(nf, dtype=torch.uint8, device="cuda") if (use_ws and nf) else False
    wsd = torch.empty(nd, dtype=torch.uint8, device="cuda") if (use_ws and nd) else False
    assert not use_ws or nf or nd

    def run():
        y = B.qeft_linear_fwd(h.desc, w, xd, ws=wsf)
        dx = B.qeft_linear_bwd_dx(h.desc, w, dyd, ws=wsd)
        dw = B.qeft_weak_grad(h.desc, dyd, xd[:, ic - k:], out_dtype=torch.float32)
        torch.cuda.synchronize()
        return y, dx, dw

    first = run()
    for _ in range(5):
        for a, b in zip(run(), first):
            assert torch.equal(a, b)


SHORT_CASES = [  # oc, ic, k, m, layer seed: found on the CPU (tests/test_oracle_linear.py) to leave the bar with fp16-rounded weights
    (8, 320, 256, 130, 14),
    (8, 640, 256, 260, 14),
]


@pytest.mark.parametrize("oc,ic,k,m,seed", SHORT_CASES)
def test_backward_dx_short_contraction(oc, ic, k, m, seed):
    """Input gradients that sum only eight terms: rounding the dequantized weights to fp16, as the tiled kernels do, puts
    single outputs of these two cases outside the per-element bar, so contractions under 64 terms run on the kernels
    that keep s (q - z) in fp32."""
    h = HostLayer(oc, ic, k, 4, 128, seed=seed)
    dy = synth.make_grad_output(m, oc, seed=m)
    dx = B.qeft_linear_bwd_dx(h.desc, h.to_device(), pad_cols(dy)[0])
    torch.cuda.synchronize()
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"dX {oc}x{ic} k{k} M{m}")


@pytest.mark.parametrize("ic,k", [(8, 0), (8, 8), (16, 8), (56, 24)])
def test_forward_short_contraction(ic, k):
    h = HostLayer(264, ic, k, 4, 128, seed=ic + k)
    w = h.to_device()
    for m in (17, 70, 260):
        x = synth.make_activations(m, ic, k, seed=m)
        y = B.qeft_linear_fwd(h.desc, w, pad_cols(x)[0])
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"fwd 264x{ic} k{k} M{m}")

