"""GPU parity on seeded random shapes: the decode forward at 1 to 16 rows (one layer, or two or three layers that share
their input in one launch) and the one-call backward, every output compared in full with the oracle's product.

The fixed cases elsewhere sit on the shapes the kernels were written for; the host-side choices between kernels (ranges
of a row per wave, waves per row, tiles per workgroup, passes over a long row, split launches) change at boundaries that
no fixed list covers.  This sweep draws rows of 8 to 29600 columns, 8 to 9000 rows, weak blocks of 8 to 256 columns,
4-bit and both 3-bit layouts from one seed, so that a wrong choice at such a boundary shows up as a wrong product.
(Twice it did: three tiles per workgroup with two passes over a row, and rows of 9 to 12 ranges split over four waves.)
Stored components are drawn on the host and bit-packed by the oracle.
"""
import numpy as np
import pytest
import torch

from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth
from parity_util import BigLayer, assert_close

pytestmark = pytest.mark.gpu


def _decode_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for case in range(n):
        bits = [4, 4, 3, "3d"][case % 4]
        r = rng.random()
        if r < 0.25:
            kq = int(rng.choice([8, 64, 128, 504, 1024, 2040, 2048, 2056, 4088, 4096, 4104]))
        elif r < 0.6:
            kq = 8 * int(rng.integers(1, 1400))
        else:
            kq = 8 * int(rng.integers(1400, 3700))
        k = int(rng.choice([8, 16, 24, 64, 128, 200, 256]))
        ic = kq + k
        oc_max = max(16, min(9000, int(30e6 // ic)))
        oc = int(rng.choice([8, 16, 24, 40, 136, 520])) if rng.random() < 0.2 else 8 * int(rng.integers(1, oc_max // 8 + 1))
        n_layers = int(rng.choice([1, 1, 1, 2, 3])) if oc * ic * 3 < 40e6 else 1
        ocs = [oc] + [max(8, 8 * int(rng.integers(1, oc // 8 + 1))) for _ in range(n_layers - 1)]
        Ms = sorted(set(int(m) for m in rng.choice(np.arange(1, 17), size=3, replace=False)) | {1})
        cases.append((case, tuple(ocs), ic, k, bits, tuple(Ms)))
    return cases


@pytest.mark.parametrize("case,ocs,ic,k,bits,Ms", _decode_cases(48, seed=2024))
def test_decode_random_shapes(case, ocs, ic, k, bits, Ms):
    Ls = [BigLayer(oc, ic, k, bits, 1000 * case + i) for i, oc in enumerate(ocs)]
    for m in Ms:
        x = synth.make_activations(m, ic, k, seed=m + case)
        xt = torch.from_numpy(x).cuda()
        if len(Ls) == 1:
            ys = [B.qeft_linear_fwd(Ls[0].desc, Ls[0].dev, xt)]
        else:
            ys = [torch.empty((m, L.oc), dtype=torch.float16, device="cuda") for L in Ls]
            B.qeft_linear_fwd_group([L.desc for L in Ls], [L.dev for L in Ls], xt, ys)
        torch.cuda.synchronize()
        for i, L in enumerate(Ls):
            assert_close(ys[i].float().cpu().numpy(), x.astype(np.float64) @ L.w64.T, f"layer {i} ({L.oc}x{ic} k{k} w{bits}) M={m}")


def _backward_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for case in range(n):
        oc = 8 * int(rng.integers(8, 400))
        kq = 128 * int(rng.integers(1, 24)) if rng.random() < 0.7 else 8 * int(rng.integers(8, 300))
        k = int(rng.choice([8, 64, 128, 256]))
        cases.append((case, oc, kq + k, k, int(rng.integers(17, 900))))
    return cases


@pytest.mark.parametrize("case,oc,ic,k,m", _backward_cases(16, seed=77))
def test_backward_in_one_call_random_shapes(case, oc, ic, k, m):
    """qeft_linear_bwd with the weak gradient's workspace alone and with room for a row split of dX."""
    L = BigLayer(oc, ic, k, 4, 5000 + case)
    x = synth.make_activations(m, ic, k, seed=case)
    dy = synth.make_grad_output(m, oc, seed=case + 1)
    dyt, xw = torch.from_numpy(dy).cuda(), torch.from_numpy(np.ascontiguousarray(x[:, ic - k:])).cuda()
    for op in (B.QEFT_OP_WEAK_GRAD, B.QEFT_OP_BWD):
        ws = torch.empty(max(B.qeft_workspace_bytes(L.desc, op, m), 16), dtype=torch.uint8, device="cuda")
        dx, dw = B.qeft_linear_bwd(L.desc, L.dev, dyt, xw, ws=ws)
        torch.cuda.synchronize()
        assert_close(dx.float().cpu().numpy(), dy.astype(np.float64) @ L.w64, f"dX {oc}x{ic} k{k} M={m}")
        assert_close(dw.float().cpu().numpy(), dy.astype(np.float64).T @ x[:, ic - k:].astype(np.float64), f"dW {oc}x{k} M={m}")


def _gemm_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for case in range(n):
        bits = [4, 4, 4, 3, "3d"][case % 5]
        r = rng.random()
        kq = 0 if r < 0.05 else (64 * int(rng.integers(1, 100)) if r < 0.6 else 8 * int(rng.integers(1, 800)))
        k = int(rng.choice([0, 8, 24, 64, 128, 192, 256, 320]))
        if kq + k < 64:
            k = 64
        if kq == 0:
            bits = 4
        oc = 8 * int(rng.integers(1, 500))
        m = int(rng.choice([17, 33, 48, 64, 100, 255, 256, 257, 300, 511, 700, 1024, 1500, 2100]))
        cases.append((case, oc, kq + k, k, bits, m))
    return cases


@pytest.mark.parametrize("case,oc,ic,k,bits,m", _gemm_cases(20, seed=5))
def test_gemm_paths_random_shapes(case, oc, ic, k, bits, m):
    """Forward and input gradient at more than 16 rows, without and with the optional workspace (split launches; the
    fp16 copy of a 3-bit layer), and the weak gradient in both output types and on a view into X."""
    L = BigLayer(oc, ic, k, bits, 100 + case)
    kq = ic - k
    x = synth.make_activations(m, ic, k, seed=case)
    dy = synth.make_grad_output(m, oc, seed=case + 1)
    xt, dyt = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    x64, dy64 = x.astype(np.float64), dy.astype(np.float64)
    yref, dxref = x64 @ L.w64.T, dy64 @ L.w64
    for ws in (False, None):      # False: no workspace; None: the binding allocates what qeft_workspace_bytes reports
        y = B.qeft_linear_fwd(L.desc, L.dev, xt, ws=ws)
        dx = B.qeft_linear_bwd_dx(L.desc, L.dev, dyt, ws=ws)
        torch.cuda.synchronize()
        assert_close(y.float().cpu().numpy(), yref, f"fwd {oc}x{ic} k{k} w{bits} M={m} ws={ws}")
        assert_close(dx.float().cpu().numpy(), dxref, f"dX {oc}x{ic} k{k} w{bits} M={m} ws={ws}")
    if k:
        dwref = dy64.T @ x64[:, kq:]
        xw = torch.from_numpy(np.ascontiguousarray(x[:, kq:])).cuda()
        for dt in (torch.float32, torch.float16):
            dw = B.qeft_weak_grad(L.desc, dyt, xw, out_dtype=dt)
            torch.cuda.synchronize()
            assert_close(dw.float().cpu().numpy(), dwref, f"dW {oc}x{k} M={m} {dt}")
        dw = B.qeft_weak_grad(L.desc, dyt, xt[:, kq:], out_dtype=torch.float32)
        torch.cuda.synchronize()
        assert_close(dw.float().cpu().numpy(), dwref, f"dW {oc}x{k} M={m} on a view into X")
