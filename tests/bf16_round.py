"""bfloat16 rounding for the tests of the opt-in reduced-precision scorer (QUOKA_SCORE_QBAR_BF16).

Rounding Q-bar to bfloat16 is this library's own approximation, not something the paper defines (its
conclusion only names a cheaper Q-bar K^T as future work), so the helper lives with the tests and not in
the oracle: a test rounds Q-bar with it and feeds the result to the oracle's unchanged scoring function.
"""
from __future__ import annotations

import numpy as np


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest bfloat16 value (8 significant bits, ties to even) of every finite float32-representable entry,
    returned as float64."""
    f = np.asarray(x, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.float64)
    flat_in, flat_out = f.reshape(-1), out.reshape(-1)
    for i, v in enumerate(flat_in):
        v = float(v)
        if v == 0.0 or not np.isfinite(v):
            flat_out[i] = v
            continue
        m, e = np.frexp(v)             # v = m * 2**e, 0.5 <= |m| < 1
        scaled = m * 256.0             # 8 significant bits: integer part in [128, 256)
        r = np.floor(scaled)
        frac = scaled - r
        if frac > 0.5 or (frac == 0.5 and int(r) % 2 == 1):
            r += 1.0
        flat_out[i] = float(np.ldexp(r / 256.0, int(e)))
    return out
