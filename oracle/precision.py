"""Mixed-precision convention of the oracle.

The paper trains in fp32 throughout (Sec. 5.1).  The bf16 workloads add one rule: matrix
operands (weights, and the activations handed across the library boundary) are bf16
values.  The oracle therefore rounds those inputs to bf16 once, round-to-nearest-even,
and afterwards computes in fp64 with no further rounding.
"""
import numpy as np


def round_to_bf16(a):
    """Round float32 values to the nearest bfloat16 (ties to even); returns float64."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    bits = a32.view(np.uint32).astype(np.uint64)
    keep_lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + keep_lsb) & np.uint64(0xFFFF0000)
    out = bits.astype(np.uint32).view(np.float32)
    nan = np.isnan(a32)
    if nan.any():
        out = np.where(nan, np.float32(np.nan), out)
    return out.astype(np.float64)
