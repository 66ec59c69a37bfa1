"""Storage precisions of the CPU oracle.  Test infrastructure (CPU oracle).

The paper does not fix an arithmetic precision.  The benchmark configurations name two policies:
everything in single/double precision ("f64" here: the oracle computes in fp64 throughout), and
"bf16 activations with fp32 master weights" ("bf16" here).  In the second policy every tensor that
the method STORES between steps -- layer outputs, back-propagated gradients, the working copy of
the weights -- holds bfloat16 values, while sums are carried in higher precision and the master
weights, momentum and weight gradients are not rounded.  The oracle follows that policy by rounding
exactly those tensors to the bfloat16 grid and doing all arithmetic in fp64.  This matters for
parity because ReLU masks and pooling winners are decisions taken on stored values: both
implementations must take them on the same numbers.

bfloat16 = the upper 16 bits of an IEEE binary32 (8 exponent bits, 7 stored mantissa bits);
rounding is to nearest, ties to the value whose last kept bit is 0.
"""
import numpy as np


def round_to_bf16(a):
    """Nearest bfloat16 value (ties to even) of every element, returned as float64."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lower = bits & 0xFFFF
    upper = bits >> 16
    round_up = (lower > 0x8000) | ((lower == 0x8000) & ((upper & 1) == 1))
    upper = upper + round_up.astype(np.uint64)
    out = (upper << 16).astype(np.uint32).view(np.float32)
    out = np.where(np.isfinite(f), out, f)
    return out.astype(np.float64).reshape(np.shape(a))


def identity(a):
    return np.asarray(a, dtype=np.float64)


def storage_rounding(precision):
    if precision == "f64":
        return identity
    if precision == "bf16":
        return round_to_bf16
    raise ValueError("unknown precision policy %r" % (precision,))
