"""Dropout + residual add + LayerNorm on rows, written out from the definitions in fp64.

TEST INFRASTRUCTURE ONLY (see oracle.py).  Shares no code with the HIP library.

The paper fuses the Dropout, Add and LayerNorm operators of the BERT encoder into
one forward and two backward kernels (Section IV-C-1, "Dropout_Add_LayerNorm
Fusion") and prints no formula; these are the operators' textbook definitions:

  forward   z = x o M c + r            (M the keep mask, c = 1 / (1 - p))
            mu = mean(z), var = mean((z - mu)^2)          (per row, biased variance)
            rstd = 1 / sqrt(var + eps)
            y = (z - mu) rstd gamma + beta
  backward  for upstream dy, with xh = (z - mu) rstd and g = dy gamma:
            dz = rstd (g - mean(g) - xh mean(g xh))        (per row)
            dr = dz,  dx = dz o M c
            dgamma = sum_rows dy xh,  dbeta = sum_rows dy

The mask is an explicit input here; how the GPU side draws it is restated in
ln_keep_mask below (the same generator, Philox4x32-10, as for the attention mask).
"""
from __future__ import annotations

import numpy as np

from . import dropout_mask as dm

LN_TAG = 0x4C4E  # third counter word of the LayerNorm mask's generator calls


def ln_keep_mask(rows: int, hidden: int, p: float, seed: int, first_row: int = 0) -> np.ndarray:
    """[rows, hidden] uint8, 1 = kept, for rows first_row .. first_row + rows - 1 of the tensor.
    Element (t, c) reads byte (c & 15) - byte c & 3 of word (c >> 2) & 3 - of the call with
    counter (c >> 4, t, LN_TAG, 0) and the seed as key; kept iff that byte >= round(256 p)."""
    t, c = np.meshgrid(np.arange(first_row, first_row + rows, dtype=np.int64),
                       np.arange(hidden, dtype=np.int64), indexing="ij")
    ctr = np.stack([c >> 4, t, np.full_like(t, LN_TAG), np.zeros_like(t)], axis=-1).astype(np.uint32)
    out = dm.philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    word = np.take_along_axis(out, ((c >> 2) & 3)[..., None], axis=-1)[..., 0]
    byte = (word >> (8 * (c & 3)).astype(np.uint32)) & np.uint32(0xFF)
    return (byte >= dm.threshold(p)).astype(np.uint8)


def fwd(x, r, gamma, beta, eps, mask=None, keep_scale=1.0):
    """Returns (y, z, mu, rstd); x, r: [T, N]; gamma, beta: [N]; mask: [T, N] or None."""
    x, r = np.asarray(x, dtype=np.float64), np.asarray(r, dtype=np.float64)
    gamma, beta = np.asarray(gamma, dtype=np.float64), np.asarray(beta, dtype=np.float64)
    t, n = x.shape
    y, z = np.zeros((t, n)), np.zeros((t, n))
    mu, rstd = np.zeros(t), np.zeros(t)
    for i in range(t):
        zi = x[i] * (mask[i] * keep_scale if mask is not None else 1.0) + r[i]
        m = zi.sum() / n
        var = ((zi - m) ** 2).sum() / n
        rs = 1.0 / np.sqrt(var + eps)
        z[i], mu[i], rstd[i] = zi, m, rs
        y[i] = (zi - m) * rs * gamma + beta
    return y, z, mu, rstd


def bwd(dy, x, r, gamma, eps, mask=None, keep_scale=1.0):
    """Returns (dx, dr, dgamma, dbeta) for the forward above (recomputed from x and r)."""
    dy = np.asarray(dy, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    _, z, mu, rstd = fwd(x, r, gamma, np.zeros_like(gamma), eps, mask, keep_scale)
    t, n = z.shape
    dx, dr = np.zeros((t, n)), np.zeros((t, n))
    dgamma, dbeta = np.zeros(n), np.zeros(n)
    for i in range(t):
        xh = (z[i] - mu[i]) * rstd[i]
        g = dy[i] * gamma
        dz = rstd[i] * (g - g.sum() / n - xh * (g * xh).sum() / n)
        dr[i] = dz
        dx[i] = dz * (mask[i] * keep_scale if mask is not None else 1.0)
        dgamma += dy[i] * xh
        dbeta += dy[i]
    return dx, dr, dgamma, dbeta
