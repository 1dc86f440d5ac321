"""Rounding to a reduced storage format, for the mixed-precision workload (bf16 activations, fp32
master weights).

bfloat16 is the upper half of an IEEE binary32: 1 sign bit, 8 exponent bits, 7 stored mantissa
bits.  round_bf16 maps every value to the nearest bfloat16 (ties to the even mantissa) and returns
it as float64, so the float64 model can be evaluated on exactly the numbers a bf16 tensor can hold.
The value is first rounded to binary32, as an fp32 accumulator would hold it.
"""
import numpy as np


def round_bf16(a):
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = (r & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(a))
