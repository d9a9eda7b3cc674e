"""qeft_weak_grad_noalloc (the entry point for callers that cannot allocate or pass a workspace) against
qeft_weak_grad on the same inputs: same kernels, so the results must be equal bit for bit; and against the oracle
to the usual bar.  Two calls in a row share the library's per-GPU scratch array, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import qeft_oracle as qo
from paper_2410_08661_amd import binding as B
from paper_2410_08661_amd import synth
from parity_util import assert_close

pytestmark = pytest.mark.gpu


def _inputs(oc, k, m, seed):
    ic = 512 + k
    x = synth.make_activations(m, ic, k, seed)
    dy = synth.make_grad_output(m, oc, seed)
    return B.make_desc(oc, ic, k, 4, 128), x[:, ic - k:], dy


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16])
def test_noalloc_equals_the_workspace_call_twice_in_a_row(dtype):
    # first a 7B-sized call that uses 8 MiB of the scratch array (4 token splits), then a smaller one (other split
    # count, ragged channel count) that finds the first call's partial sums still in the array
    for oc, k, m, seed in [(4096, 128, 4096, 1), (1032, 64, 700, 2)]:
        desc, xw, dy = _inputs(oc, k, m, seed)
        assert 0 < B.qeft_workspace_bytes(desc, B.QEFT_OP_WEAK_GRAD, m) <= 14 * 1024 * 1024
        dyd = torch.from_numpy(dy).cuda()
        xwd = torch.from_numpy(np.ascontiguousarray(xw)).cuda()
        ref_call = B.qeft_weak_grad(desc, dyd, xwd, out_dtype=dtype)
        got = torch.full((oc, k), 3.0, dtype=dtype, device="cuda")
        B.qeft_weak_grad_noalloc(desc, dyd, xwd, got)
        torch.cuda.synchronize()
        assert torch.equal(got, ref_call)
        assert_close(got.float().cpu().numpy(), qo.weak_grad(dy, xw), f"noalloc dW {oc}x{k} M{m}")
        # accumulate on top
        B.qeft_weak_grad_noalloc(desc, dyd, xwd, got, accumulate=True)
        B.qeft_weak_grad(desc, dyd, xwd, dW=ref_call, accumulate=True)
        torch.cuda.synchronize()
        assert torch.equal(got, ref_call)


def test_noalloc_rejects_what_does_not_fit():
    oc, k, m = 16320, 128, 256                               # 2 token splits x 16320 x 128 x 4 B = 15.9 MiB of partial sums
    desc = B.make_desc(oc, 512 + k, k, 4, 128)
    assert B.qeft_workspace_bytes(desc, B.QEFT_OP_WEAK_GRAD, m) > 14 * 1024 * 1024
    dy = torch.zeros((m, oc), dtype=torch.float16, device="cuda")
    xw = torch.zeros((m, k), dtype=torch.float16, device="cuda")
    dw = torch.full((oc, k), 5.0, dtype=torch.float32, device="cuda")
    with pytest.raises(B.QeftError) as e:
        B.qeft_weak_grad_noalloc(desc, dy, xw, dw)
    assert e.value.status == B.QEFT_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.all(dw == 5.0)                              # a failing call has no effect
    small = B.make_desc(64, 128, 64, 4, 128)
    with pytest.raises(B.QeftError) as e:                    # M < 64: the general kernel's case, no scratch involved
        B.qeft_weak_grad_noalloc(small, dy[:8, :64], xw[:8, :64], torch.zeros((64, 64), dtype=torch.float32, device="cuda"))
    assert e.value.status == B.QEFT_ERR_UNSUPPORTED
