"""Backward of an embedding lookup: dW[v] = sum of the output-gradient rows whose index is v.

TEST INFRASTRUCTURE ONLY (see oracle.py).  Shares no code with the HIP library.

Section IV-C-3 of the paper: in the backward of the embedding, "the output's gradient
from the same index should be accumulated to get the weight's gradient".  Exact
definition, accumulated in fp64 in token order; indices outside [0, vocab) and the
optional padding index contribute nothing.
"""
from __future__ import annotations

import numpy as np


def embedding_bwd(dy, indices, vocab: int, padding_idx: int = -1, dw_init=None):
    """dy: [T, N]; indices: [T] integers.  Returns dW [vocab, N] float64 (added onto dw_init
    if given) and counts [vocab] (how many rows went into each)."""
    dy = np.asarray(dy, dtype=np.float64)
    t, n = dy.shape
    dw = np.zeros((vocab, n)) if dw_init is None else np.array(dw_init, dtype=np.float64)
    counts = np.zeros(vocab, dtype=np.int64)
    for i in range(t):
        v = int(indices[i])
        if v < 0 or v >= vocab or v == padding_idx:
            continue
        dw[v] += dy[i]
        counts[v] += 1
    return dw, counts


def abs_sums(dy, indices, vocab: int, padding_idx: int = -1):
    """A[v] = sum of |dy rows| with index v: bounds every partial sum in any accumulation order."""
    return embedding_bwd(np.abs(np.asarray(dy, dtype=np.float64)), indices, vocab, padding_idx)[0]
