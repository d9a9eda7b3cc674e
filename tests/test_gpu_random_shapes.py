"""GPU parity on seeded random shapes: output / input channels, weak-block widths and token counts drawn from
lists that straddle every dispatch boundary (matrix-vector kernels up to 16 tokens, tiled kernels above; whole and
ragged 64-column stages; layers without quantized or without weak columns), for 4-bit codes and both 3-bit layouts.
Forward always; input gradient and weak-block gradient at GEMM sizes.  Same bar as everywhere (parity_util)."""
import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth
from parity_util import HostLayer, assert_close, pad_cols

pytestmark = pytest.mark.gpu

OCS = [8, 16, 24, 40, 72, 136, 200, 264, 520, 1000]
KQS = [8, 64, 120, 128, 136, 256, 384, 504, 512, 640, 1024, 1160, 2048]
KS = [0, 8, 16, 24, 64, 72, 128, 192, 256]
MS = [1, 2, 3, 4, 5, 8, 13, 16, 17, 40, 70, 130, 260]


def _case(i):
    rng = np.random.default_rng(1000 + i)
    bits, dense = [(4, False), (3, False), (3, True)][i % 3]
    oc, kq, k = int(rng.choice(OCS)), int(rng.choice(KQS)), int(rng.choice(KS))
    if rng.random() < 0.1:
        kq = 0
    if kq + k == 0:
        k = 64
    ms = [int(m) for m in rng.choice(MS, size=3, replace=False)]
    return oc, kq, k, bits, dense, ms


@pytest.mark.parametrize("i", range(45))
def test_random_shape(i):
    oc, kq, k, bits, dense, ms = _case(i)
    ic = kq + k
    h = HostLayer(oc, ic, k, bits, 128, seed=i, dense=dense)
    w = h.to_device()
    what = f"oc={oc} ic={ic} k={k} bits={bits} dense={dense}"
    for m in ms:
        x = synth.make_activations(m, ic, k, seed=m + i)
        xv, _ = pad_cols(x)
        y = B.qeft_linear_fwd(h.desc, w, xv)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"{what} fwd M{m}")
        if m <= 16:
            continue
        dy = synth.make_grad_output(m, oc, seed=m)
        dyv, _ = pad_cols(dy)
        dx = B.qeft_linear_bwd_dx(h.desc, w, dyv)
        torch.cuda.synchronize()
        assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"{what} dX M{m}")
        if k:
            xw, _ = pad_cols(x[:, kq:])
            dw = B.qeft_weak_grad(h.desc, dyv, xw, out_dtype=torch.float32)
            torch.cuda.synchronize()
            assert_close(dw.cpu().numpy(), qo.weak_grad(dy, x[:, kq:]), f"{what} dW M{m}")


def _tail_case(i):
    """Launches of 160 - 420 tiles whose last round leaves at most half of an XCD's compute units busy and whose
    contraction is long enough that the library splits it, for those tiles only, when given the optional workspace."""
    rng = np.random.default_rng(2000 + i)
    while True:
        tn, tm = int(rng.integers(3, 40)), int(rng.integers(4, 12))
        n = tn * 256 - int(rng.choice([0, 8, 64, 120, 200]))     # channels along the tiled dimension (ragged last tile)
        m = tm * 256 - int(rng.choice([0, 1, 77, 255]))
        k = int(rng.choice([0, 64, 128, 256]))
        depth = int(rng.choice([2048, 2560, 3072, 4096]))        # length of the contraction
        ic = (n - k) // 128 * 128 + k                            # dX: about n input channels, whole groups
        fwd, dx = B.make_desc(n, depth + k, k, 4, 128), B.make_desc(depth, ic, k, 4, 128)
        if tn * tm >= 160 and B.qeft_workspace_bytes(fwd, B.QEFT_OP_FWD, m) > 0 and B.qeft_workspace_bytes(dx, B.QEFT_OP_BWD_DX, m) > 0:
            return n, m, k, depth, ic


@pytest.mark.parametrize("i", range(4))
def test_random_shape_with_split_last_round(i):
    n, m, k, depth, ic = _tail_case(i)
    # forward: n output channels, contraction over depth quantized + k weak input channels
    h = HostLayer(n, depth + k, k, 4, 128, seed=i)
    w = h.to_device()
    x = synth.make_activations(m, depth + k, k, seed=i)
    y = B.qeft_linear_fwd(h.desc, w, torch.from_numpy(x).cuda())        # the binding allocates the workspace
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), qo.linear_fwd(h.w64, x), f"fwd {n}x{depth + k} k={k} M{m}")
    del h, w, x, y
    # input gradient: ic input channels, contraction over depth weight rows
    h = HostLayer(depth, ic, k, 4, 128, seed=i + 50)
    w = h.to_device()
    dy = synth.make_grad_output(m, depth, seed=i)
    dx = B.qeft_linear_bwd_dx(h.desc, w, torch.from_numpy(dy).cuda())
    torch.cuda.synchronize()
    assert_close(dx.cpu().numpy(), qo.linear_bwd_dx(h.w64, dy), f"dX {depth}x{ic} k={k} M{m}")
