"""Keep-mask of attention-probability dropout, written out element by element.

TEST INFRASTRUCTURE ONLY (see oracle.py).  Shares no code with the HIP library.

The paper's training runs use BERT's dropout on the attention probabilities
(the model of Section V-A); it does not say how the fused attention kernel
draws it.  The reading taken here: the random bits come from a counter-based
generator, so that forward and backward (and any implementation) can
regenerate the same mask from (seed, position) alone.  The generator is
Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel random
numbers: as easy as 1, 2, 3", SC 2011): a 128-bit counter, a 64-bit key,
128 output bits per call.

Definition of the mask.  For the sequence that starts at packed row r0, head h,
query q and key k (both counted from the start of the sequence):

  * the 4x4 block (Q4, K4) = (q >> 2, k >> 2) owns one generator call with
    counter words (K4, Q4, r0, h) and key words (seed & 0xffffffff, seed >> 32);
  * the call's 16 output bytes are B[x][y] = byte y (little endian) of output
    word x; element (q, k) uses x = ((q & 3) - (k >> 3)) & 3 and
    y = ((k & 3) - (q >> 3)) & 3 - within a block a one-to-one map of the 16
    elements onto the 16 bytes;
  * the element is KEPT iff B[x][y] >= t, where t = round(256 p) clamped to
    [0, 255]; the dropout probability actually applied is t / 256 and kept
    probabilities are multiplied by 256 / (256 - t).
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_LO = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(counter: np.ndarray, key) -> np.ndarray:
    """counter: [..., 4] uint32; key: two uint32 values.  Returns [..., 4] uint32."""
    c = [np.asarray(counter[..., i], dtype=np.uint64) for i in range(4)]
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c[0]  # 32 x 32 -> 64 bit products, exact in uint64
        p1 = _M1 * c[2]
        c = [(p1 >> _S32) ^ c[1] ^ np.uint64(k0), p1 & _LO,
             (p0 >> _S32) ^ c[3] ^ np.uint64(k1), p0 & _LO]
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack(c, axis=-1).astype(np.uint32)


def threshold(p: float) -> int:
    """t = round(256 p), clamped to [0, 255]."""
    if not (0.0 <= p < 1.0):
        raise ValueError("dropout probability must be in [0, 1)")
    return min(255, max(0, int(np.floor(256.0 * p + 0.5))))


def keep_scale(p: float) -> float:
    return 256.0 / (256.0 - threshold(p))


def random_bytes(r0: int, heads: int, n_q: int, n_k: int, seed: int) -> np.ndarray:
    """The byte every (head, q, k) element of one sequence compares with t: [heads, n_q, n_k] uint8."""
    h, q, k = np.meshgrid(np.arange(heads, dtype=np.int64), np.arange(n_q, dtype=np.int64),
                          np.arange(n_k, dtype=np.int64), indexing="ij")
    ctr = np.stack([k >> 2, q >> 2, np.full_like(q, r0), h], axis=-1).astype(np.uint32)
    out = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))
    x = ((q & 3) - (k >> 3)) & 3
    y = ((k & 3) - (q >> 3)) & 3
    word = np.take_along_axis(out, x[..., None], axis=-1)[..., 0]
    return ((word >> (8 * y).astype(np.uint32)) & np.uint32(0xFF)).astype(np.uint8)


def keep_masks(cu_seqlens, heads: int, p: float, seed: int):
    """Per sequence a [heads, L, L] uint8 array (1 = kept)."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    t = threshold(p)
    masks = []
    for i in range(len(cu) - 1):
        n = int(cu[i + 1] - cu[i])
        masks.append((random_bytes(int(cu[i]), heads, n, n, seed) >= t).astype(np.uint8))
    return masks
