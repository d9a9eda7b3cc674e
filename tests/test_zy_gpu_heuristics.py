"""Perf-informational: the host-side choices between kernels, on shapes OFF the Llama-2 grid.

Two choices are made from time models fitted to the Llama-2 shapes: several 16-token passes of the matrix-vector
kernel instead of a GEMM that would fill a fraction of the compute units (forward without workspace, 16 < M <= 256),
and splitting the contraction of some or all tiles over the optional workspace.  These tests time the library's
choice and the alternative that the boundary lets a caller force (the passes as calls on 16-row slices; the call
without the workspace) with HIP events and require the choice to be at most 10 % slower than that alternative.
No numerics here (the parity tests cover every path); a failure means a heuristic needs refitting, not a wrong
result.  Timings on a shared machine wobble, so a miss is measured a second time, and only a miss of more than 25 %
fails the test; one between 10 % and 25 % is reported as an expected-failure note with the figures.  The file is named
to be collected after the parity tests: a run that stops at the first failure has then compared every result first.
"""
import pytest
import torch

from paper_2410_08661_amd import binding as B

pytestmark = pytest.mark.gpu

SLACK, HARD = 1.10, 1.25


def _judge(measure, what):
    """measure() -> (library's time, alternative's time); informational between SLACK and HARD, failing beyond."""
    t_lib, t_alt = measure()
    if t_lib > SLACK * t_alt:
        t_lib, t_alt = measure()          # once more before believing it
    print(f"\n{what}: library {t_lib:.1f} us, alternative {t_alt:.1f} us")
    assert t_lib <= HARD * t_alt, f"{what}: {t_lib:.1f} us against {t_alt:.1f} us"
    if t_lib > SLACK * t_alt:
        pytest.xfail(f"{what}: {t_lib:.1f} us against {t_alt:.1f} us (more than 10 % slower than the alternative)")


def _layer(oc, ic, k, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    d = B.make_desc(oc, ic, k, 4, 128)
    w = B.Weight(d)
    w.qweight.random_(-2**31, 2**31 - 1, generator=gen)
    w.scales.copy_((torch.rand(w.scales.shape, generator=gen, device="cuda") * 0.008 + 0.004).half())
    w.zeros.copy_(torch.randint(0, 16, w.zeros.shape, generator=gen, device="cuda").half())
    w.weak.copy_((torch.randn(w.weak.shape, generator=gen, device="cuda") * 0.02).half())
    return d, w, gen


def _us(fn, n=20, repeats=3):
    """Best of `repeats` event timings of n back-to-back calls, in microseconds per call."""
    for _ in range(3):
        fn()
    best = float("inf")
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) * 1e3 / n)
    return best


@pytest.mark.parametrize("oc,ic", [(6144, 6144), (2560, 7168)])
@pytest.mark.parametrize("m", [48, 96, 320])
def test_passes_or_gemm_without_workspace(oc, ic, m):
    d, w, gen = _layer(oc, ic, 128, oc + m)
    x = torch.randn((m, ic), generator=gen, device="cuda").half()
    y = torch.empty((m, oc), dtype=torch.float16, device="cuda")
    def passes():
        for r in range(0, m, 16):
            B.qeft_linear_fwd(d, w, x[r:r + 16], y[r:r + 16], ws=False)
    _judge(lambda: (_us(lambda: B.qeft_linear_fwd(d, w, x, y, ws=False)), _us(passes)),
           f"forward {oc}x{ic} M={m} without workspace against {(m + 15) // 16} passes of 16 rows")


@pytest.mark.parametrize("oc,ic,m", [(6144, 6144, 48), (6144, 6144, 320), (6144, 6144, 2816), (2560, 7168, 320), (7168, 2560, 1536)])
def test_workspace_never_costs_more_than_ten_percent(oc, ic, m):
    """With the optional workspace the library may split tiles (all of them when they are few, the last round's when
    it is sparse); a caller who passes one must not lose by it."""
    d, w, gen = _layer(oc, ic, 128, oc + ic + m)
    x = torch.randn((m, ic), generator=gen, device="cuda").half()
    dy = (torch.randn((m, oc), generator=gen, device="cuda") * 0.01).half()
    y = torch.empty((m, oc), dtype=torch.float16, device="cuda")
    dx = torch.empty((m, ic), dtype=torch.float16, device="cuda")
    for name, op, call in (("forward", B.QEFT_OP_FWD, lambda ws: B.qeft_linear_fwd(d, w, x, y, ws=ws)),
                           ("dX", B.QEFT_OP_BWD_DX, lambda ws: B.qeft_linear_bwd_dx(d, w, dy, dx, ws=ws))):
        n = B.qeft_workspace_bytes(d, op, m)
        if n == 0:
            continue                     # no split planned for this launch: both calls are the same
        ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        _judge(lambda: (_us(lambda: call(ws)), _us(lambda: call(False))), f"{name} {oc}x{ic} M={m} with the workspace against without")
