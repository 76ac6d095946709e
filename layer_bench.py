"""Times the convolution entry points of the C ABI (resist_conv2d_forward / _dgrad / _wgrad) on the layer
shapes of a benchmark configuration, one layer at a time:

    python3 layer_bench.py [--config cfg2|cfg4|cfg5_bf16] [--dtype f32|bf16] [--reps N] [--layers a,b] [fwd] [dgrad] [wgrad]

Prints microseconds per call (HIP events around `reps` back-to-back calls, so launch overhead is included)
the rate in algorithmic TFLOP/s (2*N*P*Q*K*C*R*S per call) and in algorithmic GB/s (the three tensors once)."""
import argparse
import ctypes as C

import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from paper_2107_00961_amd import binding as B  # noqa: E402

# name, input H (= W), C, K, filter size, stride, pad
LAYERS = {
    "cfg2": (128, [("s1_3x3", 32, 64, 64, 3, 1, 1), ("s2_3x3", 16, 128, 128, 3, 1, 1), ("s3_3x3", 8, 256, 256, 3, 1, 1),
                   ("s4_3x3", 4, 512, 512, 3, 1, 1), ("s2_first", 32, 64, 128, 3, 2, 1), ("s3_first", 16, 128, 256, 3, 2, 1),
                   ("s4_first", 8, 256, 512, 3, 2, 1), ("s3_shortcut", 16, 128, 256, 1, 2, 0),
                   # the 1x1 layers of the bottleneck blocks
                   ("s1_1x1_in", 32, 256, 64, 1, 1, 0), ("s1_1x1_out", 32, 64, 256, 1, 1, 0),
                   ("s2_1x1_in", 16, 512, 128, 1, 1, 0), ("s2_1x1_out", 16, 128, 512, 1, 1, 0),
                   ("s3_1x1_in", 8, 1024, 256, 1, 1, 0), ("s3_1x1_out", 8, 256, 1024, 1, 1, 0),
                   ("s4_1x1_in", 4, 2048, 512, 1, 1, 0), ("s4_1x1_out", 4, 512, 2048, 1, 1, 0)]),
    # the full model at CIFAR shape in bf16 (same layer shapes as cfg2)
    "cfg5_bf16": (128, [("s1_3x3", 32, 64, 64, 3, 1, 1), ("s2_3x3", 16, 128, 128, 3, 1, 1), ("s3_3x3", 8, 256, 256, 3, 1, 1),
                        ("s4_3x3", 4, 512, 512, 3, 1, 1)]),
    "cfg4": (64, [("s1_1x1_in", 56, 256, 64, 1, 1, 0), ("s1_3x3", 56, 64, 64, 3, 1, 1), ("s1_1x1_out", 56, 64, 256, 1, 1, 0),
                  ("s2_1x1_in", 28, 512, 128, 1, 1, 0), ("s2_3x3", 28, 128, 128, 3, 1, 1), ("s2_1x1_out", 28, 128, 512, 1, 1, 0),
                  ("s3_1x1_in", 14, 1024, 256, 1, 1, 0), ("s3_3x3", 14, 256, 256, 3, 1, 1), ("s3_1x1_out", 14, 256, 1024, 1, 1, 0),
                  ("s4_1x1_in", 7, 2048, 512, 1, 1, 0), ("s4_3x3", 7, 512, 512, 3, 1, 1), ("s4_1x1_out", 7, 512, 2048, 1, 1, 0),
                  ("s2_3x3_first", 56, 128, 128, 3, 2, 1), ("s2_shortcut", 56, 256, 512, 1, 2, 0)]),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2", choices=sorted(LAYERS))
    ap.add_argument("--dtype", default=None, choices=["f32", "bf16"])
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--layers", default="", help="comma-separated layer names (default: all)")
    ap.add_argument("which", nargs="*", default=["fwd", "dgrad", "wgrad"])
    args = ap.parse_args()
    which = args.which or ["fwd", "dgrad", "wgrad"]
    dtype = args.dtype or ("f32" if args.config == "cfg2" else "bf16")
    td, code = (torch.bfloat16, 1) if dtype == "bf16" else (torch.float32, 0)
    batch, layers = LAYERS[args.config]
    keep = set(args.layers.split(",")) if args.layers else None
    lib = B.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.reps

    for name, H, Cc, K, R, stride, pad in layers:
        if keep is not None and name not in keep:
            continue
        P = (H + 2 * pad - R) // stride + 1
        x = torch.randn(batch, H, H, Cc, device="cuda").to(td)
        w = torch.randn(K, R, R, Cc, device="cuda").to(td)
        y = torch.empty(batch, P, P, K, device="cuda", dtype=td)
        dy = torch.randn(batch, P, P, K, device="cuda").to(td)
        dx = torch.empty_like(x)
        dw = torch.empty(K, R, R, Cc, device="cuda")
        sh = B._conv_shape(batch, H, H, Cc, K, R, stride, pad, code)
        ws = B._conv_ws(sh)
        flops = 2.0 * batch * P * P * K * Cc * R * R
        es = 2 if dtype == "bf16" else 4
        nbytes = {"fwd": es * (x.numel() + y.numel() + w.numel()), "dgrad": es * (x.numel() + y.numel() + w.numel()),
                  "wgrad": es * (x.numel() + y.numel()) + 4 * w.numel()}
        calls = {"fwd": lambda: lib.resist_conv2d_forward(C.byref(sh), x.data_ptr(), w.data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel(), stream),
                 "dgrad": lambda: lib.resist_conv2d_dgrad(C.byref(sh), dy.data_ptr(), w.data_ptr(), dx.data_ptr(), ws.data_ptr(), ws.numel(), stream),
                 "wgrad": lambda: lib.resist_conv2d_wgrad(C.byref(sh), dy.data_ptr(), x.data_ptr(), dw.data_ptr(), ws.data_ptr(), ws.numel(), stream)}
        cells = []
        for k in which:
            t = timed(calls[k])
            cells.append(f"{k} {t * 1e3:7.1f} us {flops / t / 1e9:6.1f} TFLOP/s {nbytes[k] / t / 1e6:5.0f} GB/s")
        print(f"{name:12s} {dtype} rows={batch * P * P:6d} C={Cc:4d} K={K:4d} {R}x{R}/{stride} | " + " | ".join(cells), flush=True)


if __name__ == "__main__":
    main()
