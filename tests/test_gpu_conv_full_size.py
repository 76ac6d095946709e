"""GPU parity at the benchmark's full sizes: every distinct convolution shape of the CIFAR-shaped
(fp32 and bf16) and ImageNet-shaped (bf16) networks at the benchmark batch size, in the launch
configuration bench.py times: forward, data gradient and weight gradient, every element against the
full-tensor oracle (a second or two per layer on the GPU machine's host cores), and sampled outputs
against the point-wise form of the definition."""
import numpy as np
import pytest
import torch

import paper_2107_00961_amd as R
from oracle import layers as L
from resist_inputs import get_config, model_blocks

pytestmark = pytest.mark.gpu

NPTS = 48


def _shapes(cfg_name):
    """Distinct (H, C, K, R, stride, pad) of the block convolutions of the configuration's network."""
    cfg = get_config(cfg_name)
    m = cfg["model"]
    h = m["in_h"] if m["stem_kind"] == 0 else m["in_h"] // 4
    out = []
    for blk in model_blocks(m):
        s = blk["stride"]
        if m["block_kind"] == 0:
            convs = [(h, blk["c_in"], blk["width"], 3, s, 1), (h // s, blk["width"], blk["c_out"], 3, 1, 1)]
        else:
            convs = [(h, blk["c_in"], blk["width"], 1, 1, 0), (h, blk["width"], blk["width"], 3, s, 1),
                     (h // s, blk["width"], blk["c_out"], 1, 1, 0)]
        if blk["has_ds"]:
            convs.append((h, blk["c_in"], blk["c_out"], 1, s, 0))
        for c in convs:
            if c not in out:
                out.append(c)
        h //= s
    return cfg["batch"], out


def _cases():
    cases = []
    # cfg5_bf16: the CIFAR-shaped layers in bf16 run on the eight-wave tiles (operands requested two chunks ahead)
    for name, dt in (("cfg2", torch.float32), ("cfg4", torch.bfloat16), ("cfg5_bf16", torch.bfloat16)):
        batch, shapes = _shapes(name)
        cases += [pytest.param(name, dt, batch, s, id=f"{name}-H{s[0]}-C{s[1]}-K{s[2]}-R{s[3]}-s{s[4]}") for s in shapes]
    return cases


@pytest.mark.parametrize("name,dt,N,shape", _cases())
def test_full_size_conv(name, dt, N, shape):
    H, C, K, RS, st, pad = shape
    print(f"{name} N={N} shape={shape} dtype={dt}", flush=True)
    P = (H + 2 * pad - RS) // st + 1
    g = torch.Generator(device="cuda").manual_seed(1234)
    x = torch.randn((N, H, H, C), generator=g, device="cuda").to(dt)
    w = (torch.randn((K, RS, RS, C), generator=g, device="cuda") / float(np.sqrt(C * RS * RS))).to(dt)
    dy = torch.randn((N, P, P, K), generator=g, device="cuda").to(dt)
    dyw = (dy.float() / float(np.sqrt(N * P * P))).to(dt)          # keeps weight-gradient sums O(1)
    y = R.conv2d_forward(x, w, st, pad)
    dx = R.conv2d_dgrad(dy, w, (N, H, H, C), st, pad)
    dw = R.conv2d_wgrad(dyw, x, (K, RS, RS, C), st, pad)
    torch.cuda.synchronize()
    xh, wh, dyh, dywh = (t.float().cpu().numpy() for t in (x, w, dy, dyw))
    yh, dxh, dwh = y.float().cpu().numpy(), dx.float().cpu().numpy(), dw.cpu().numpy()
    rng = np.random.default_rng(5)
    # bf16 outputs carry half a bfloat16 ulp on top of the fp32 accumulation error
    rtol, atol = (2.0 ** -8, 1e-5) if dt == torch.bfloat16 else (1e-4, 1e-5)

    def check(got, want, what):
        err = np.abs(got - want)
        tol = atol + rtol * np.abs(want)
        assert np.all(err <= tol), f"{what} {name} {shape}: worst {np.max(err / tol):.2f} x tolerance"

    pts = [(rng.integers(N), rng.integers(P), rng.integers(P), rng.integers(K)) for _ in range(NPTS)]
    pts += [(0, 0, 0, 0), (N - 1, P - 1, P - 1, K - 1), (N - 1, 0, P - 1, K // 2)]
    check(np.array([yh[p] for p in pts]), L.conv2d_fwd_points(xh, wh, st, pad, pts), "fwd")
    pts = [(rng.integers(N), rng.integers(H), rng.integers(H), rng.integers(C)) for _ in range(NPTS)]
    pts += [(0, 0, 0, 0), (N - 1, H - 1, H - 1, C - 1), (N // 2, H - 1, 0, C // 2)]
    check(np.array([dxh[p] for p in pts]), L.conv2d_dgrad_points(dyh, wh, st, pad, pts), "dgrad")
    pts = [(rng.integers(K), rng.integers(RS), rng.integers(RS), rng.integers(C)) for _ in range(NPTS // 2)]
    pts += [(0, 0, 0, 0), (K - 1, RS - 1, RS - 1, C - 1)]
    rtol, atol = 1e-4, 1e-5                                           # weight gradients are fp32 in both modes
    check(np.array([dwh[p] for p in pts]), L.conv2d_wgrad_points(dywh, xh, st, pad, RS, RS, pts), "wgrad")
    # every element of all three results against the full-tensor oracle (NCHW, float64, a second or two per layer)
    xc, wc, dyc = xh.transpose(0, 3, 1, 2), wh.transpose(0, 3, 1, 2), dyh.transpose(0, 3, 1, 2)
    rtol, atol = (2.0 ** -8, 1e-5) if dt == torch.bfloat16 else (1e-4, 1e-5)
    check(yh.transpose(0, 3, 1, 2), L.conv2d_fwd(xc, wc, st, pad), "fwd, all elements")
    check(dxh.transpose(0, 3, 1, 2), L.conv2d_dgrad(dyc, wc, (N, C, H, H), st, pad), "dgrad, all elements")
    rtol, atol = 1e-4, 1e-5
    # the weight gradient: every element, through the split reduction
    dw_ref = L.conv2d_wgrad(dywh.transpose(0, 3, 1, 2), xh.transpose(0, 3, 1, 2), (K, C, RS, RS), st, pad)   # [K][C][R][S]
    check(dwh.transpose(0, 3, 1, 2), dw_ref, "wgrad, all elements")


def test_conv_1x1_at_the_size_limit():
    """Maximum sizes: an activation tensor of 2.05e9 bytes, just under the 2 GiB that the kernels' 32-bit
    byte offsets can reach (larger shapes are refused when the plan is made).  A 1x1 convolution 512 <-> 16
    channels over 61 x 128 x 128 pixels: the forward pass reads that tensor, the data gradient writes one,
    the weight gradient reduces over its 999 424 rows.  Forward and data gradient are compared on the
    first and last 1024 rows and 2048 rows in between (a 1x1 convolution treats every pixel on its own, so the
    oracle is run on those rows as a batch of one-pixel images), the weight gradient over the whole tensors."""
    N, H, W, C, K = 61, 128, 128, 512, 16
    M = N * H * W
    assert 2 ** 31 - 2 ** 27 < M * C * 4 < 2 ** 31
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    x = torch.randn((N, H, W, C), device="cuda", generator=g)
    w = torch.randn((K, 1, 1, C), device="cuda", generator=g) / np.sqrt(C)
    dy = torch.randn((N, H, W, K), device="cuda", generator=g)
    w_o = w.cpu().numpy().transpose(0, 3, 1, 2)                      # [K, C, 1, 1]
    rng = np.random.default_rng(3)
    rows = np.concatenate([np.arange(1024), np.arange(M - 1024, M), rng.integers(1024, M - 1024, 2048)])
    rows_d = torch.from_numpy(rows).cuda()

    print("forward", flush=True)
    y = R.conv2d_forward(x, w, 1, 0)
    torch.cuda.synchronize()
    xs = x.view(M, C)[rows_d].cpu().numpy()
    want = L.conv2d_fwd(xs[:, :, None, None], w_o, 1, 0)[:, :, 0, 0]
    got = y.view(M, K)[rows_d].cpu().numpy()
    assert np.all(np.abs(got - want) <= 1e-5 + 1e-4 * np.abs(want)), f"forward: max error {np.max(np.abs(got - want)):.3e}"
    del y

    print("data gradient", flush=True)
    dx = R.conv2d_dgrad(dy, w, (N, H, W, C), 1, 0)
    torch.cuda.synchronize()
    dys = dy.view(M, K)[rows_d].cpu().numpy()
    want = L.conv2d_dgrad(dys[:, :, None, None], w_o, (len(rows), C, 1, 1), 1, 0)[:, :, 0, 0]
    got = dx.view(M, C)[rows_d].cpu().numpy()
    assert np.all(np.abs(got - want) <= 1e-5 + 1e-4 * np.abs(want)), f"data gradient: max error {np.max(np.abs(got - want)):.3e}"
    del dx

    print("weight gradient", flush=True)
    dw = R.conv2d_wgrad(dy, x, (K, 1, 1, C), 1, 0)
    torch.cuda.synchronize()
    want = L.conv2d_wgrad(dy.view(M, K, 1, 1).cpu().numpy(), x.view(M, C, 1, 1).cpu().numpy(), (K, C, 1, 1), 1, 0)
    got = dw.cpu().numpy().transpose(0, 3, 1, 2)
    # a sum of 999 424 products in fp32, split over workgroups and added in a fixed order: errors of ~1e-6 of the
    # typical magnitude of an entry (~1000); entries near zero are held to that scale, not to their own size
    tol = 1e-4 * np.abs(want) + 1e-5 * np.max(np.abs(want))
    assert np.all(np.abs(got - want) <= tol), f"weight gradient: max error {np.max(np.abs(got - want)):.3e} of {np.max(np.abs(want)):.3e}"
