"""Padded <-> unpadded storage, written out from the definitions.

TEST INFRASTRUCTURE ONLY (see oracle.py).  Shares no code with the HIP library.

The paper's unpadded storage (Section IV-A-1) keeps only the valid tokens of a
[batch, max_seq_len] input, batch and sequence dimensions merged, plus a
prefix-sum array (batch_offset) of the tokens per sequence.  Section IV-B-2
names the steps that go from one format to the other:
  * nonzero_indices: the positions where input_mask is non-zero;
  * gather: keep the rows at those positions (padded -> unpadded);
  * batch_offset generation;
and Section IV-A-1 the way back before the pooler: scatter (unpadded -> padded).
The paper does not say what scatter leaves in the padding rows; the reading
here is zeros (rows nobody owns must not hold stale data).

Everything is plain loops over rows; exact (no floating-point arithmetic).
"""
from __future__ import annotations

import numpy as np


def unpad_indices(input_mask):
    """input_mask: [B, S] integers.  Returns
    nonzero_indices [n] int32 - flat positions b*S+s with input_mask[b, s] != 0, ascending;
    inverse [B*S] int32      - for each flat position its rank among those, or -1 for padding;
    cu_seqlens [B+1] int32   - prefix sums of the number of non-zero entries per row."""
    m = np.asarray(input_mask)
    assert m.ndim == 2
    nb, s = m.shape
    idx, inv, cu = [], [-1] * (nb * s), [0]
    for b in range(nb):
        for t in range(s):
            if m[b, t] != 0:
                inv[b * s + t] = len(idx)
                idx.append(b * s + t)
        cu.append(len(idx))
    return (np.array(idx, dtype=np.int32), np.array(inv, dtype=np.int32), np.array(cu, dtype=np.int32))


def gather_rows(padded, nonzero_indices):
    """padded: [B*S, ...]; returns the rows at nonzero_indices, in that order."""
    padded = np.asarray(padded)
    out = np.empty((len(nonzero_indices),) + padded.shape[1:], dtype=padded.dtype)
    for j, r in enumerate(nonzero_indices):
        out[j] = padded[int(r)]
    return out


def scatter_rows(packed, nonzero_indices, padded_rows):
    """Inverse of gather_rows: row j of `packed` goes to row nonzero_indices[j] of a
    [padded_rows, ...] array whose other rows are zero."""
    packed = np.asarray(packed)
    out = np.zeros((padded_rows,) + packed.shape[1:], dtype=packed.dtype)
    for j, r in enumerate(nonzero_indices):
        out[int(r)] = packed[j]
    return out
