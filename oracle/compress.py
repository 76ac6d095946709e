"""Oracle: b-bit compression of communicated parameters and reassembly from the compressed
copies -- TEST INFRASTRUCTURE ONLY.

Appendix "ResIST and Quantization/Sparse Gradients" (Table 9): every parameter that travels between
the workers and the server is compressed to b bits, b = 8 ... 4.  The paper does not say which
quantiser it used.  Reading taken here: the plain uniform min-max quantiser, applied to each named
tensor of a block on its own (a convolution filter, a BN vector, the FC matrix ...):

    lo = min w, hi = max w, L = 2^b - 1, delta = (hi - lo) / L
    code = round_half_even((w - lo) / delta)   in {0..L}      (delta = 0: every code is 0)
    w'   = lo + code * delta

The code is an integer decided by floating point, so the decision is taken in the precision of the
stored parameters (fp32: subtraction, division and rounding each in IEEE single precision, delta
itself the fp32 quotient).  Everything after the decision -- the decoded value and the mean over
the sub-ResNets that hold a block (Sec. 2.3) -- is float64 here.
Pins: tests/test_oracle_compress.py (arithmetic progression whose codes are known in closed form,
brute-force nearest level in float64, half-step error bound, end points, constant tensors,
reassembly invariants).
"""
import numpy as np


def levels(bits):
    if not 2 <= int(bits) <= 8:
        raise ValueError("bits must be in 2..8")
    return (1 << int(bits)) - 1


def quantize_tensor(w, bits):
    """w: array of float32 values.  Returns (codes uint8 of w's shape, lo float32, delta float32)."""
    w = np.asarray(w, np.float32)
    L = np.float32(levels(bits))
    lo = np.float32(w.min())
    hi = np.float32(w.max())
    delta = np.float32(np.float32(hi - lo) / L)
    if delta == 0:
        return np.zeros(w.shape, np.uint8), lo, delta
    t = (w - lo).astype(np.float32) / delta          # fp32 subtraction, fp32 division
    codes = np.rint(t.astype(np.float32))             # ties to even
    codes = np.clip(codes, 0, float(L))
    return codes.astype(np.uint8), lo, delta


def dequantize_tensor(codes, lo, delta):
    return np.float64(lo) + np.asarray(codes, np.float64) * np.float64(delta)


def quantize_block(tensors, bits):
    """tensors: {name: float32 array} -> {name: (codes, lo, delta)}."""
    return {name: quantize_tensor(a, bits) for name, a in tensors.items()}


def aggregate_quantized(global_params, sub_blocks, sub_q):
    """Reassembly (Sec. 2.3) when the sub-ResNets' parameters arrive compressed.
    sub_q[s][key][name] = (codes, lo, delta).  Every global tensor becomes the mean, over the
    sub-ResNets that hold its block, of the decoded copies (ascending s); one holder: the decoded
    copy; no holder: the old value."""
    B = max(global_params.keys())
    out = {}
    for key, tensors in global_params.items():
        holders = [s for s in range(len(sub_blocks)) if key in (-1, B) or key in sub_blocks[s]]
        out[key] = {}
        for name, old in tensors.items():
            if not holders:
                out[key][name] = np.array(old, copy=True)
                continue
            acc = np.zeros(np.shape(old), np.float64)
            for s in holders:
                acc = acc + dequantize_tensor(*sub_q[s][key][name])
            out[key][name] = acc / float(len(holders))
    return out
