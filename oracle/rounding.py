"""Storage-type rounding used by the oracle (test infrastructure).

The paper is silent on numeric precision.  The reading taken here: tensors that
live in memory between operators are held in the configuration's storage type
(bf16 or fp32) and every operator computes in higher precision from those
stored values.  The oracle therefore computes in fp64 and rounds at the stated
points with the two functions below (round-to-nearest, ties-to-even).
"""
import numpy as np


def round_f32(x):
    """Nearest fp32 value of each fp64 element, returned as fp64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def round_bf16(x):
    """Nearest bfloat16 value (8 exponent bits, 7 fraction bits) as fp64.

    Works directly on the fp64 bit pattern so the result is a single correct
    rounding of the fp64 input: keep the top 7 of the 52 fraction bits, i.e.
    round at bit 45, ties to even.  Inputs below the bf16 normal range are
    flushed through fp32 first (never reached by the workloads here).
    """
    x = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    bits = x.view(np.uint64)
    drop = np.uint64(45)
    lsb = (bits >> drop) & np.uint64(1)
    bias = np.uint64((1 << 44) - 1) + lsb
    rounded = ((bits + bias) >> drop) << drop
    out = rounded.view(np.float64).copy()
    tiny = np.abs(x) < 2.0 ** -126
    if np.any(tiny):
        out[tiny] = _bf16_via_f32(x[tiny])
    bad = ~np.isfinite(x)
    if np.any(bad):
        out[bad] = x[bad]
    return out.reshape(x.shape)


def _bf16_via_f32(x):
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = f.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = ((b + np.uint32(0x7FFF) + lsb) >> np.uint32(16)) << np.uint32(16)
    return r.view(np.float32).astype(np.float64)


def identity(x):
    """No rounding (used when a caller wants the unrounded fp64 value)."""
    return np.asarray(x, dtype=np.float64)


STORAGE = {"bf16": round_bf16, "fp32": round_f32, "fp64": identity}
