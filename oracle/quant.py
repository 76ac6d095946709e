"""Oracle: rounding to bfloat16 storage -- TEST INFRASTRUCTURE ONLY.

The ImageNet-shaped benchmark configuration stores activations and convolution operands as
bfloat16 (8 significand bits, fp32's exponent range) while sums stay in fp32.  This module is the
definition of that storage rounding for the oracle: a real number goes to the nearest fp32 and
then to the nearest bfloat16, ties to even, i.e. the upper 16 bits of the fp32 pattern after adding
0x7FFF plus the lowest kept bit.
Pins (tests/test_oracle_quant.py): hand-computed ties and neighbours, idempotence, monotonicity,
the error bound 2^-9 relative, a tensor library's own bfloat16 conversion as third opinion.
"""
import numpy as np


def round_bf16(a):
    """float array -> float64 array whose values are all representable in bfloat16."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    keep_lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = (u + np.uint64(0x7FFF) + keep_lsb) & np.uint64(0xFFFF0000)
    nan = np.isnan(f)
    out = r.astype(np.uint32).view(np.float32).astype(np.float64)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(a))


def identity(a):
    return a
