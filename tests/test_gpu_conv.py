"""GPU parity: the convolution kernels, through the C ABI, against the oracle's direct
convolution on the same seeded tensors (several tiles, ragged tails, both strides)."""
import numpy as np
import pytest
import torch

import paper_2107_00961_amd as R
from oracle import layers as L
from tests.gpu_util import assert_close

pytestmark = pytest.mark.gpu

#         N   H   W   C    K   R st pad
CASES = [(2, 16, 16, 16, 16, 3, 1, 1),      # tiny config's block shape
         (3, 12, 12, 64, 128, 3, 2, 1),     # stride 2, ragged M = 108
         (4, 16, 16, 64, 64, 3, 1, 1),      # several M tiles
         (2, 8, 8, 64, 256, 1, 1, 0),       # 1x1
         (2, 8, 8, 64, 128, 1, 2, 0),       # 1x1 stride 2 (downsample shortcut)
         (3, 10, 10, 32, 64, 1, 1, 0),      # stem-as-GEMM shape
         (2, 6, 6, 48, 80, 3, 1, 1),        # channel counts that are not multiples of the K-chunk
         (32, 32, 32, 64, 256, 3, 1, 1),    # large enough for the 128x128 tile
         (2, 8, 8, 512, 512, 3, 1, 1),      # 128x128 weight-gradient tile
         (5, 14, 14, 32, 32, 3, 2, 1),      # stride 2 with odd output size 7
         (2, 12, 12, 16, 32, 5, 1, 2),      # 5x5
         (2, 14, 14, 16, 32, 5, 2, 2),      # 5x5 stride 2: three and two taps per parity class
         (1, 9, 9, 16, 16, 7, 1, 3),        # 7x7
         (2, 16, 16, 8, 16, 7, 2, 3),       # 7x7 stride 2 pad 3 (the ImageNet stem's filter geometry)
         (2, 10, 18, 32, 32, 3, 1, 1),      # images that are not square
         (3, 12, 20, 16, 32, 3, 2, 1),      # ... stride 2 (parity classes of 6 x 10 pixels)
         (2, 6, 14, 32, 64, 1, 1, 0),       # ... 1x1
         (4, 1, 1, 32, 64, 1, 1, 0),        # one pixel per image: four GEMM rows
         (1, 3, 3, 16, 16, 3, 1, 0),        # one output pixel in all
         (3, 2, 2, 16, 16, 3, 2, 1)]        # 2x2 input, stride 2: one output pixel per image, three of four parity classes empty of taps


def _tensors(case, seed=0):
    N, H, W, C, K, RS, st, pad = case
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    w = (rng.standard_normal((K, C, RS, RS), dtype=np.float32) / np.sqrt(C * RS * RS)).astype(np.float32)
    P, Q = (H + 2 * pad - RS) // st + 1, (W + 2 * pad - RS) // st + 1
    dy = rng.standard_normal((N, K, P, Q), dtype=np.float32)
    return x, w, dy


def _nhwc(a):
    return torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 3, 1))).cuda()


@pytest.mark.parametrize("case", CASES)
def test_conv_forward(case):
    print("case", case, flush=True)
    x, w, _ = _tensors(case)
    st, pad = case[6], case[7]
    y = R.conv2d_forward(_nhwc(x), _nhwc(w), st, pad)
    torch.cuda.synchronize()
    want = L.conv2d_fwd(x, w, st, pad)
    assert_close(y.cpu().numpy().transpose(0, 3, 1, 2), want, f"conv fwd {case}")


@pytest.mark.parametrize("case", CASES)
def test_conv_dgrad(case):
    print("case", case, flush=True)
    x, w, dy = _tensors(case, 1)
    N, H, W, C, K, RS, st, pad = case
    dx = R.conv2d_dgrad(_nhwc(dy), _nhwc(w), (N, H, W, C), st, pad)
    torch.cuda.synchronize()
    want = L.conv2d_dgrad(dy, w, x.shape, st, pad)
    assert_close(dx.cpu().numpy().transpose(0, 3, 1, 2), want, f"conv dgrad {case}")


@pytest.mark.parametrize("case", CASES)
def test_conv_wgrad(case):
    print("case", case, flush=True)
    x, w, dy = _tensors(case, 2)
    N, H, W, C, K, RS, st, pad = case
    # keep the sums O(1) so the absolute floor of the bound means what it means for real gradients:
    # an fp32 sum of L products of O(1) terms carries an absolute error ~ sqrt(L) * 2^-24 * sqrt(L)
    dy = (dy / np.sqrt(dy.shape[0] * dy.shape[2] * dy.shape[3])).astype(np.float32)
    dw = R.conv2d_wgrad(_nhwc(dy), _nhwc(x), (K, RS, RS, C), st, pad)
    torch.cuda.synchronize()
    want = L.conv2d_wgrad(dy, x, w.shape, st, pad)
    assert_close(dw.cpu().numpy().transpose(0, 3, 1, 2), want, f"conv wgrad {case}")


# ---- bf16 operands, fp32 accumulation ---------------------------------------------------------
# Inputs are bfloat16 numbers, so the oracle's float64 result is the exact convolution of what the
# kernel reads.  Outputs stored as bfloat16 carry half a bfloat16 ulp (2^-9 relative, 2^-8 of the
# value's power of two) on top of the fp32 accumulation error; weight gradients are fp32.
BF16_CASES = [c for c in CASES if c[3] % 8 == 0 and c[4] % 8 == 0]


def _bf16_tensors(case, seed):
    x, w, dy = _tensors(case, seed)
    r = lambda a: torch.from_numpy(a).to(torch.bfloat16)
    return r(x), r(w), r(dy)


def _nhwc_t(t):
    return t.permute(0, 2, 3, 1).contiguous().cuda()


def _f64(t):
    return t.to(torch.float64).numpy()


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_forward_bf16(case):
    print("case", case, flush=True)
    x, w, _ = _bf16_tensors(case, 3)
    st, pad = case[6], case[7]
    y = R.conv2d_forward(_nhwc_t(x), _nhwc_t(w), st, pad)
    torch.cuda.synchronize()
    assert y.dtype == torch.bfloat16
    want = L.conv2d_fwd(_f64(x), _f64(w), st, pad)
    assert_close(y.cpu().to(torch.float64).numpy().transpose(0, 3, 1, 2), want, f"bf16 conv fwd {case}",
                 rtol=2.0 ** -8, atol=1e-5)


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_dgrad_bf16(case):
    print("case", case, flush=True)
    x, w, dy = _bf16_tensors(case, 4)
    N, H, W, C, K, RS, st, pad = case
    dx = R.conv2d_dgrad(_nhwc_t(dy), _nhwc_t(w), (N, H, W, C), st, pad)
    torch.cuda.synchronize()
    assert dx.dtype == torch.bfloat16
    want = L.conv2d_dgrad(_f64(dy), _f64(w), tuple(x.shape), st, pad)
    assert_close(dx.cpu().to(torch.float64).numpy().transpose(0, 3, 1, 2), want, f"bf16 conv dgrad {case}",
                 rtol=2.0 ** -8, atol=1e-5)


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_wgrad_bf16(case):
    print("case", case, flush=True)
    x, w, dy = _bf16_tensors(case, 5)
    N, H, W, C, K, RS, st, pad = case
    dy = (dy.to(torch.float32) / float(np.sqrt(dy.shape[0] * dy.shape[2] * dy.shape[3]))).to(torch.bfloat16)
    dw = R.conv2d_wgrad(_nhwc_t(dy), _nhwc_t(x), (K, RS, RS, C), st, pad)
    torch.cuda.synchronize()
    assert dw.dtype == torch.float32
    want = L.conv2d_wgrad(_f64(dy), _f64(x), tuple(w.shape), st, pad)
    assert_close(dw.cpu().numpy().transpose(0, 3, 1, 2), want, f"bf16 conv wgrad {case}")


# ---- the stem convolution: implicit GEMM straight from the [N,C,H,W] fp32 image ----------------------------
#              N  C   H   W   K  R st pad
STEM_CASES = [(4, 3, 16, 16, 16, 3, 1, 1),       # the tiny configuration's stem
              (5, 3, 32, 32, 64, 3, 1, 1),       # CIFAR-shaped: four output rows per tile
              (3, 3, 40, 40, 16, 7, 2, 3),       # 7x7 stride 2: 20 x 20 outputs, five rows per tile
              (2, 3, 224, 224, 64, 7, 2, 3),     # ImageNet-shaped: one 112-pixel row per tile
              (2, 3, 18, 30, 32, 3, 1, 1),       # rectangular, 32 output channels (one tile of channels)
              (2, 4, 12, 12, 96, 5, 2, 2),       # four input channels, 96 output channels (64 + 32), 5x5
              (1, 1, 9, 9, 16, 3, 1, 0),         # one channel, no padding
              (2, 3, 26, 134, 48, 3, 1, 1),      # 134 output columns: tiles of 67 columns (rows not a multiple of 4 wide)
              (1, 3, 8, 256, 16, 3, 1, 1),       # two tiles of 128 columns along a row that is staged in 16-byte pieces
              (1, 3, 6, 268, 16, 3, 1, 1)]       # four tiles of 67 columns: every tile starts at another offset mod 4


def _stem_tensors(case, seed, bf16):
    N, C, H, W, K, RS, st, pad = case
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    w = (rng.standard_normal((K, C, RS, RS), dtype=np.float32) / np.sqrt(C * RS * RS)).astype(np.float32)
    P, Q = (H + 2 * pad - RS) // st + 1, (W + 2 * pad - RS) // st + 1
    dy = (rng.standard_normal((N, K, P, Q), dtype=np.float32) / np.sqrt(N * P * Q)).astype(np.float32)
    if bf16:   # bfloat16 numbers, so the float64 result is the exact convolution of what the kernel multiplies
        x, w, dy = (torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy() for a in (x, w, dy))
    return x, w, dy


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", STEM_CASES)
def test_stem_conv_forward(case, bf16):
    print("case", case, "bf16" if bf16 else "f32", flush=True)
    x, w, _ = _stem_tensors(case, 6, bf16)
    st, pad = case[6], case[7]
    y = R.stem_conv2d_forward(torch.from_numpy(x).cuda(), _nhwc(w), st, pad, bf16=bf16)
    torch.cuda.synchronize()
    want = L.conv2d_fwd(x, w, st, pad)
    got = y.cpu().to(torch.float64).numpy().transpose(0, 3, 1, 2)
    if bf16:
        assert_close(got, want, f"bf16 stem fwd {case}", rtol=2.0 ** -8, atol=1e-5)
    else:
        assert_close(got, want, f"stem fwd {case}")


@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("case", STEM_CASES)
def test_stem_conv_wgrad(case, bf16):
    print("case", case, "bf16" if bf16 else "f32", flush=True)
    x, w, dy = _stem_tensors(case, 7, bf16)
    N, C, H, W, K, RS, st, pad = case
    dyd = _nhwc(dy)
    if bf16:
        dyd = dyd.to(torch.bfloat16)
    dw = R.stem_conv2d_wgrad(dyd, torch.from_numpy(x).cuda(), (K, RS, RS, C), st, pad)
    torch.cuda.synchronize()
    want = L.conv2d_wgrad(dy, x, w.shape, st, pad)
    assert_close(dw.cpu().numpy().transpose(0, 3, 1, 2), want, f"stem wgrad {case} {'bf16' if bf16 else 'f32'}")


def test_stem_conv_rejects_bad_shapes():
    x = torch.zeros((1, 5, 8, 8), device="cuda")
    with pytest.raises(R.ResistError):
        R.stem_conv2d_forward(x, torch.zeros((16, 3, 3, 5), device="cuda"), 1, 1)        # five input channels
    with pytest.raises(R.ResistError):
        R.stem_conv2d_forward(torch.zeros((1, 3, 8, 8), device="cuda"), torch.zeros((24, 3, 3, 3), device="cuda"), 1, 1)   # K = 24


def test_conv_rejects_bad_shapes():
    x = torch.zeros((1, 4, 4, 6), device="cuda")
    w = torch.zeros((8, 3, 3, 6), device="cuda")
    with pytest.raises(R.ResistError):
        R.conv2d_forward(x, w, 1, 1)          # C not a multiple of 4
    x = torch.zeros((1, 5, 5, 8), device="cuda")
    w = torch.zeros((8, 3, 3, 8), device="cuda")
    with pytest.raises(R.ResistError):
        R.conv2d_dgrad(torch.zeros((1, 3, 3, 8), device="cuda"), w, (1, 5, 5, 8), 2, 1)   # odd size, stride 2
