"""GPU: the weight-gradient entry point that allocates nothing (resist_conv2d_wgrad_static), through
the C ABI: same bits as resist_conv2d_wgrad and the fp32 bound against the oracle's direct
convolution, on two calls in a row, the second with a smaller input (the static scratch keeps the
first call's partial sums)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2107_00961_amd as R
from oracle import layers as L
from tests.gpu_util import assert_close

pytestmark = pytest.mark.gpu

#         N   H   W   C    K   R st pad     both use split partial sums; the second is smaller
CALLS = [(16, 16, 16, 64, 64, 3, 1, 1),
         (8, 16, 16, 32, 64, 3, 2, 1)]


def _nhwc(a):
    return torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 3, 1))).cuda()


def _case(case, seed):
    N, H, W, C, K, RS, st, pad = case
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    P, Q = (H + 2 * pad - RS) // st + 1, (W + 2 * pad - RS) // st + 1
    dy = (rng.standard_normal((N, K, P, Q), dtype=np.float32) / np.sqrt(N * P * Q)).astype(np.float32)
    return x, dy


@pytest.mark.parametrize("bf16", [False, True])
def test_wgrad_static_two_calls_in_a_row(bf16):
    assert R.conv2d_wgrad_static_limit() == 32 << 20
    for i, case in enumerate(CALLS):
        print("call", i, case, "bf16" if bf16 else "f32", flush=True)
        N, H, W, C, K, RS, st, pad = case
        x, dy = _case(case, 10 + i)
        xd, dyd = _nhwc(x), _nhwc(dy)
        if bf16:
            xd, dyd = xd.to(torch.bfloat16), dyd.to(torch.bfloat16)
            x = xd.float().cpu().numpy().transpose(0, 3, 1, 2)      # the oracle convolves what the kernel reads
            dy = dyd.float().cpu().numpy().transpose(0, 3, 1, 2)
        dw = torch.full((K, RS, RS, C), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        R.conv2d_wgrad_static(dyd, xd, dw, st, pad)
        torch.cuda.synchronize()
        ref = R.conv2d_wgrad(dyd, xd, (K, RS, RS, C), st, pad)
        torch.cuda.synchronize()
        assert torch.equal(dw, ref)                                  # same kernels, same order: same bits
        want = L.conv2d_wgrad(dy, x, (K, C, RS, RS), st, pad)
        assert_close(dw.cpu().numpy().transpose(0, 3, 1, 2), want, f"static wgrad call {i} {case}")


def test_wgrad_static_rejects_oversized_partial_sums():
    """A 512 x 512 3x3 filter over 2048 pixels takes the 128x128 tile and 5 splits: 47 MB of partial
    sums, more than the 32 MiB array.  The call must refuse before any launch and leave dw alone."""
    N, H, W, C, K, RS, st, pad = 128, 4, 4, 512, 512, 3, 1, 1
    sh = R.binding._conv_shape(N, H, W, C, K, RS, st, pad, 0)
    n = ctypes.c_int64()
    assert R.lib().resist_conv2d_workspace_bytes(ctypes.byref(sh), ctypes.byref(n)) == 0
    assert n.value > R.conv2d_wgrad_static_limit()
    x = torch.zeros((N, H, W, C), dtype=torch.float32, device="cuda")
    dy = torch.zeros((N, H, W, K), dtype=torch.float32, device="cuda")
    dw = torch.full((K, RS, RS, C), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(R.ResistError, match="static scratch"):
        R.conv2d_wgrad_static(dy, x, dw, st, pad)
    torch.cuda.synchronize()
    assert bool((dw == 7.0).all())
