"""Round-to-nearest-even from float64 to the bfloat16 grid (oracle side).

bfloat16 is the upper 16 bits of an IEEE binary32: 1 sign, 8 exponent and 7
stored fraction bits.  A float64 has 52 fraction bits, so a normal bfloat16
keeps the top 7 of them; the remaining 45 decide the rounding.  Results that
would be bfloat16 subnormals (magnitude below 2**-126) go through float32
first, which is exact enough for tensors that never get that small.
"""
from __future__ import annotations

import numpy as np

_DROP = 45                      # fraction bits of a float64 below bfloat16's last place
_HALF = np.uint64(1 << (_DROP - 1))
_MASK = np.uint64((1 << _DROP) - 1)


def round_to_bf16(x) -> np.ndarray:
    """Return float64 values that lie exactly on the bfloat16 grid."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    bits = x.view(np.uint64).copy()
    low = bits & _MASK
    lsb = (bits >> np.uint64(_DROP)) & np.uint64(1)
    trunc = bits & ~_MASK
    up = (low > _HALF) | ((low == _HALF) & (lsb == np.uint64(1)))
    rounded = trunc + np.where(up, np.uint64(1 << _DROP), np.uint64(0))
    out = rounded.view(np.float64).reshape(x.shape)
    mag = np.abs(x)
    tiny = mag < 2.0 ** -126
    if tiny.any():
        f32 = x.astype(np.float32)
        b32 = f32.view(np.uint32).astype(np.uint64)
        low32 = b32 & np.uint64(0xFFFF)
        lsb32 = (b32 >> np.uint64(16)) & np.uint64(1)
        up32 = (low32 > np.uint64(0x8000)) | ((low32 == np.uint64(0x8000)) & (lsb32 == np.uint64(1)))
        r32 = ((b32 & np.uint64(0xFFFF0000)) + np.where(up32, np.uint64(0x10000), np.uint64(0))).astype(np.uint32)
        out = np.where(tiny, r32.view(np.float32).astype(np.float64).reshape(x.shape), out)
    big = mag >= 2.0 ** 128
    if big.any():                # beyond bfloat16's largest finite value
        out = np.where(big & np.isfinite(x), np.sign(x) * np.inf, out)
    return np.where(np.isfinite(x), out, x)
