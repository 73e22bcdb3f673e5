"""bfloat16 <-> float32 on the host, for the oracle.  TEST INFRASTRUCTURE.

bfloat16 is the upper 16 bits of an IEEE-754 binary32.  Widening is exact.
Narrowing rounds to nearest, ties to even, on the 16 discarded bits; a NaN
stays a (quiet) NaN.  bf16 buffers are carried as ``numpy.uint16`` arrays.

The paper does not fix a dtype; for bf16 the per-op rule used throughout is
widen both operands to fp32, add once in fp32, round once to bf16 - what a
rank does when it reduces a bf16 chunk received over the wire.
"""

import numpy as np


def bf16_to_f32(u16):
    u16 = np.asarray(u16, dtype=np.uint16)
    return (u16.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(x):
    """Round-to-nearest-even narrowing; returns uint16 bit patterns."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    keep = bits >> np.uint32(16)
    rest = bits & np.uint32(0xFFFF)
    half = np.uint32(0x8000)
    up = (rest > half) | ((rest == half) & ((keep & np.uint32(1)) == 1))
    out = keep + up.astype(np.uint32)          # carry may run into the exponent: correct
    nan = (bits & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    out = np.where(nan, keep | np.uint32(0x0040), out)
    return out.astype(np.uint16)


def bf16_add(a_u16, b_u16):
    """rnd(a + b) for bf16 operands given as uint16 bit patterns."""
    with np.errstate(over="ignore", invalid="ignore"):
        return f32_to_bf16(bf16_to_f32(a_u16) + bf16_to_f32(b_u16))
