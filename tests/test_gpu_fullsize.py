"""GPU parity at the full benchmark sizes (the Llama-2 7B / 13B / 70B layer shapes), in the
launch configuration bench.py times.  The oracle cannot form whole products at these sizes
in a test, so it computes sampled outputs one by one (unpack the row, dequantize, dot), and
the whole output is additionally checked for finiteness and against the samples' scale.

Stored components are drawn on the host (uniform codes, realistic scales, integer zero-points)
and bit-packed by the oracle; nothing the oracle consumes comes from the GPU.
"""
import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth
from parity_util import REL

pytestmark = pytest.mark.gpu

N_SAMPLES = 192


class BigLayer:
    def __init__(self, oc, ic, k, bits, seed):
        # bits "3d": 3-bit codes in the dense layout
        dense = bits == "3d"
        nbits = 3 if dense else bits
        self.oc, self.ic, self.k, self.bits, self.g = oc, ic, k, bits, 128
        self.lay = qo.layout(oc, ic, k, nbits, 128, dense=dense)
        self.kq = self.lay["kq"]
        codes, self.scales, self.zeros = synth.make_codes(oc, self.kq, self.lay["n_groups"], nbits, seed)
        if dense:
            self.qweight = qo.pack_codes_dense3(codes, self.lay["row_stride_words"])
        else:
            self.qweight = qo.pack_codes(codes, bits, self.lay["row_stride_words"])
        del codes
        self.weak = (np.random.default_rng(seed).standard_normal((oc, k), dtype=np.float32) * 0.02).astype(np.float16)
        self.desc = B.make_desc(oc, ic, k, nbits, 128, layout=B.QEFT_LAYOUT_DENSE3 if dense else B.QEFT_LAYOUT_CANONICAL)
        w = B.Weight(self.desc)
        ng = self.lay["n_groups"]
        w.qweight.copy_(torch.from_numpy(self.qweight.view(np.int32)))
        w.scales[:, :ng].copy_(torch.from_numpy(self.scales))
        w.zeros[:, :ng].copy_(torch.from_numpy(self.zeros))
        w.weak.copy_(torch.from_numpy(self.weak))
        self.dev = w

    def args(self):
        return (self.qweight, self.scales, self.zeros, self.weak, self.kq, self.bits, self.g)


def _pairs(n_rows, n_cols, seed, edge_cols=()):
    r = np.random.default_rng(seed)
    rows = r.integers(0, n_rows, N_SAMPLES)
    cols = r.integers(0, n_cols, N_SAMPLES)
    # always include the corners and the given boundary columns
    extra = [(0, 0), (n_rows - 1, n_cols - 1), (0, n_cols - 1), (n_rows - 1, 0)]
    extra += [(int(rows[i]), int(c)) for i, c in enumerate(edge_cols) if 0 <= c < n_cols]
    return extra + list(zip(rows.tolist(), cols.tolist()))


def _check(actual_t, pairs, ref, what):
    a_all = actual_t.float().cpu().numpy()
    assert np.all(np.isfinite(a_all)), f"{what}: non-finite output"
    a = np.array([a_all[i, j] for i, j in pairs], dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    worst = float(np.max(np.abs(a - ref) - REL * (np.abs(ref) + rms)))
    assert worst <= 0, f"{what}: sampled element off by {worst:.3e} beyond the bar (rms {rms:.3e})"
    fro = float(np.linalg.norm(a - ref) / np.linalg.norm(ref))
    assert fro <= REL, f"{what}: sampled relative error {fro:.3e}"
    # the whole output has the magnitude the samples predict (catches tiles never written)
    got_rms = float(np.sqrt(np.mean(a_all.astype(np.float64) ** 2)))
    assert 0.5 * rms <= got_rms <= 2.0 * rms, f"{what}: output rms {got_rms:.3e} vs sampled {rms:.3e}"


DECODE = [  # config, shapes, k, bits list, M list
    (2, synth.LLAMA_7B, 128, [4], [1, 8, 40, 100]),     # 40, 100: between the matrix-vector kernels and the GEMM
    (3, synth.LLAMA_13B, 128, [3, 4], [1, 3, 5, 16]),
    (3, synth.LLAMA_13B, 128, ["3d"], [1, 5, 16]),      # the dense 3-bit layout
    (5, synth.LLAMA_70B, 256, [4], [1, 4]),
]
DECODE_CASES = [(cfg, si, s, k, b, Ms) for cfg, shapes, k, bl, Ms in DECODE for si, s in enumerate(shapes) for b in bl]


@pytest.mark.parametrize("cfg,si,shape,k,bits,Ms", DECODE_CASES)
def test_decode_forward_full_size(cfg, si, shape, k, bits, Ms):
    oc, ic = shape
    seed = synth.seed_for(cfg, si)
    L = BigLayer(oc, ic, k, bits, seed)
    for m in Ms:
        x = synth.make_activations(m, ic, k, seed + m)
        y = B.qeft_linear_fwd(L.desc, L.dev, torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        pairs = _pairs(m, oc, seed + m)
        ref = qo.fwd_samples(*L.args(), x, pairs)
        _check(y, pairs, ref, f"cfg{cfg} fwd {oc}x{ic} b{bits} M{m}")


GROUPS = [  # the launches bench.py times: layers that share their input, one launch each
    ("q/k/v", [(4096, 4096)] * 3, 128),
    ("gate/up", [(11008, 4096)] * 2, 128),
]


@pytest.mark.parametrize("name,shapes,k", GROUPS)
def test_decode_group_full_size(name, shapes, k):
    ic = shapes[0][1]
    Ls = [BigLayer(oc, ic, k, 4, synth.seed_for(2, 10 + i)) for i, (oc, _) in enumerate(shapes)]
    x = synth.make_activations(1, ic, k, synth.seed_for(2, 20))
    ys = B.qeft_linear_fwd_group([L.desc for L in Ls], [L.dev for L in Ls], torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    for i, (L, y) in enumerate(zip(Ls, ys)):
        pairs = _pairs(1, L.oc, 30 + i)
        _check(y, pairs, qo.fwd_samples(*L.args(), x, pairs), f"{name} layer {i} {L.oc}x{ic} M1 (one launch)")


@pytest.mark.parametrize("m", [1, 4096])
def test_irregular_out_proj_full_size(m):
    """The 7B output projection with its weak columns left at arbitrary channels."""
    oc = ic = 4096
    k = 128
    L = BigLayer(oc, ic, k, 4, synth.seed_for(2, 40))
    weak_idx = np.sort(np.random.default_rng(41).permutation(ic)[:k])
    perm = qo.stored_order(ic, weak_idx)
    x = synth.make_activations(m, ic, 0, synth.seed_for(2, 42))
    x[:, weak_idx] *= 20.0
    xs = np.ascontiguousarray(x[:, perm])          # what the stored layer multiplies (gathered on the host for the samples)
    y = B.qeft_linear_fwd_irregular(L.desc, L.dev, torch.from_numpy(perm).cuda(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    pairs = _pairs(m, oc, 43)
    _check(y, pairs, qo.fwd_samples(*L.args(), xs, pairs), f"irregular fwd 4096x4096 M{m}")
    if m > 1:
        dy = synth.make_grad_output(m, oc, 44)
        dx = B.qeft_linear_bwd_dx_irregular(L.desc, L.dev, torch.from_numpy(perm).cuda(), torch.from_numpy(dy).cuda())
        torch.cuda.synchronize()
        pairs = _pairs(m, ic, 45, edge_cols=[int(weak_idx[0]), int(weak_idx[-1]), 0, ic - 1])
        # sample (row, original channel): the stored column of channel c is inv[c]
        inv = np.empty(ic, dtype=np.int64)
        inv[perm] = np.arange(ic)
        ref = qo.bwd_dx_samples(*L.args(), dy, [(r, int(inv[c])) for r, c in pairs])
        _check(dx, pairs, ref, f"irregular dX 4096x4096 M{m}")


TRAIN = [(4, synth.LLAMA_7B, 128, 4096), (5, synth.LLAMA_70B, 256, 2048),
         (3, synth.LLAMA_13B, 128, 4096)]   # the 13B shapes: 320 / 864 tiles, whose last round is split (4 and 2 ways)
TRAIN_CASES = [(cfg, si, s, k, m) for cfg, shapes, k, m in TRAIN for si, s in enumerate(shapes)]


@pytest.mark.parametrize("cfg,si,shape,k,m", TRAIN_CASES)
def test_finetune_step_full_size(cfg, si, shape, k, m):
    oc, ic = shape
    seed = synth.seed_for(cfg, si)
    L = BigLayer(oc, ic, k, 4, seed)
    x = synth.make_activations(m, ic, k, seed)
    dy = synth.make_grad_output(m, oc, seed)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    kq = ic - k

    y = B.qeft_linear_fwd(L.desc, L.dev, xd)
    torch.cuda.synchronize()
    pairs = _pairs(m, oc, seed + 1)
    _check(y, pairs, qo.fwd_samples(*L.args(), x, pairs), f"cfg{cfg} fwd {oc}x{ic} M{m}")
    del y

    dx = B.qeft_linear_bwd_dx(L.desc, L.dev, dyd)
    torch.cuda.synchronize()
    # sample both sides of the quantized / weak boundary and of a group boundary
    pairs = _pairs(m, ic, seed + 2, edge_cols=[kq - 1, kq, kq + 1, ic - 1, 127, 128, kq - 128, kq - 129])
    _check(dx, pairs, qo.bwd_dx_samples(*L.args(), dy, pairs), f"cfg{cfg} dX {oc}x{ic} M{m}")
    del dx

    dw = B.qeft_weak_grad(L.desc, dyd, xd[:, kq:], out_dtype=torch.float32)
    torch.cuda.synchronize()
    pairs = _pairs(oc, k, seed + 3)
    _check(dw, pairs, qo.weak_grad_samples(dy, x[:, kq:], pairs), f"cfg{cfg} dW {oc}x{k} M{m}")
