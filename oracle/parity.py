"""Error measures used when a result is compared with the oracle's.

TEST INFRASTRUCTURE ONLY, like the rest of this package: tests, the smoke check and the
benchmark's parity / cpu_baseline leg may import this; the HIP library and its binding never do.
"""
from __future__ import annotations

import numpy as np

O_TOL = 5e-3      # outputs: max-abs
G_TOL = 1e-2      # gradients: relative, see gradient_errors
G_FLOOR = 0.1     # smallest scale a sequence's gradient error is measured against


def gradient_errors(got: np.ndarray, want: np.ndarray, cu_seqlens, floor: float = G_FLOOR):
    """(worst sequence, Frobenius): the largest, over the sequences, of max-abs error over a
    sequence's rows / max |reference| over the same rows - floored at `floor`, because a
    gradient that vanishes by exact cancellation (one token, constant V) leaves only the
    16-bit rounding of O inside D = rowsum(dO * O), which has to be measured against
    something - and ||got - want||_F / ||want||_F over the whole tensor.  Measuring every
    sequence on its own scale keeps short sequences (large gradients) from setting the bar
    for long ones (small gradients) in a mixed batch."""
    worst = 0.0
    for i in range(len(cu_seqlens) - 1):
        a, e = int(cu_seqlens[i]), int(cu_seqlens[i + 1])
        if e > a:
            worst = max(worst, float(np.abs(got[a:e] - want[a:e]).max() / max(np.abs(want[a:e]).max(), floor)))
    fro = float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)) if want.size else 0.0
    return worst, fro
