"""16-bit payloads with the special patterns of the two formats mixed in: infinities,
quiet and signalling NaNs with payloads and signs, subnormals, the largest finite
values and values whose sums leave the format.  Input generation only (no arithmetic
of the method); used by the CPU and GPU edge-payload tests."""
from __future__ import annotations

import numpy as np

SPECIAL = {
    "bf16": [0x7F80, 0xFF80,            # +inf, -inf
             0x7FC0, 0xFFC0, 0x7F81, 0xFFFF, 0x7FA5,   # quiet / signalling NaNs, payloads, signs
             0x0001, 0x8001, 0x007F, 0x0080,           # smallest / largest subnormal, smallest normal
             0x7F7F, 0xFF7F, 0x7F00,                   # largest finite values
             0x0000, 0x8000],                          # signed zeros
    "f16": [0x7C00, 0xFC00,
            0x7E00, 0xFE00, 0x7C01, 0xFFFF, 0x7D55,
            0x0001, 0x8001, 0x03FF, 0x0400,
            0x7BFF, 0xFBFF, 0x7800,
            0x0000, 0x8000],
}


def special_payload(shape, fmt, seed, density=0.03, body=None):
    """uint16 patterns: `body` (or small normal numbers of the format) with a fraction
    `density` of the entries replaced by the special patterns above, at seeded places."""
    rng = np.random.default_rng(seed)
    n = int(np.prod(shape))
    if body is None:
        small = rng.integers(-64, 65, size=n).astype(np.float32) / np.float32(8.0)
        if fmt == "f16":
            out = small.astype(np.float16).view(np.uint16).copy()
        else:
            out = (small.view(np.uint32) >> np.uint32(16)).astype(np.uint16)     # exact: few significant bits
    else:
        out = np.ascontiguousarray(body, dtype=np.uint16).reshape(-1).copy()
    where = rng.random(n) < density
    out[where] = rng.choice(np.array(SPECIAL[fmt], dtype=np.uint16), size=int(where.sum()))
    return out.reshape(shape)
