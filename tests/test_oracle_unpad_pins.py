"""Pins for oracle/unpad.py: closed forms, numpy's own nonzero / take / cumsum as a second
opinion, and the round trips that define gather and scatter as inverses.  No GPU."""
import numpy as np
import pytest

from oracle import unpad

RNG = np.random.default_rng(170)


def prefix_mask(lengths, s):
    m = np.zeros((len(lengths), s), dtype=np.int32)
    for i, n in enumerate(lengths):
        m[i, :n] = 1
    return m


def test_hand_worked_example():
    # two sequences of a [2, 4] input: tokens at (0,0), (0,1), (1,0), (1,1), (1,2)
    m = np.array([[1, 1, 0, 0], [1, 1, 1, 0]])
    idx, inv, cu = unpad.unpad_indices(m)
    assert idx.tolist() == [0, 1, 4, 5, 6]
    assert inv.tolist() == [0, 1, -1, -1, 2, 3, 4, -1]
    assert cu.tolist() == [0, 2, 5]


def test_closed_forms():
    idx, inv, cu = unpad.unpad_indices(np.ones((3, 5), dtype=np.int32))
    assert idx.tolist() == list(range(15)) and inv.tolist() == list(range(15)) and cu.tolist() == [0, 5, 10, 15]
    idx, inv, cu = unpad.unpad_indices(np.zeros((3, 5), dtype=np.int32))
    assert idx.size == 0 and (inv == -1).all() and cu.tolist() == [0, 0, 0, 0]
    lengths = [3, 0, 7, 1]
    idx, inv, cu = unpad.unpad_indices(prefix_mask(lengths, 7))
    assert cu.tolist() == np.concatenate([[0], np.cumsum(lengths)]).tolist()
    assert idx.tolist() == [i * 7 + t for i, n in enumerate(lengths) for t in range(n)]


def test_against_numpy_on_arbitrary_masks():
    # masks with holes and values other than 1: "non-zero" is the criterion
    m = RNG.integers(-1, 3, size=(9, 33)) * (RNG.random((9, 33)) < 0.6)
    idx, inv, cu = unpad.unpad_indices(m)
    assert np.array_equal(idx, np.flatnonzero(m.ravel()))
    assert np.array_equal(cu, np.concatenate([[0], np.cumsum((m != 0).sum(axis=1))]))
    assert np.array_equal(inv[idx], np.arange(len(idx)))
    assert (inv[m.ravel() == 0] == -1).all()


def test_gather_and_scatter_are_inverse_on_the_valid_rows():
    m = prefix_mask([4, 1, 6, 0, 3], 6)
    idx, inv, cu = unpad.unpad_indices(m)
    x = RNG.integers(0, 2 ** 16, size=(30, 8)).astype(np.uint16)
    g = unpad.gather_rows(x, idx)
    assert np.array_equal(g, np.take(x, idx, axis=0))
    back = unpad.scatter_rows(g, idx, 30)
    assert np.array_equal(back, x * (m.ravel() != 0)[:, None])          # padding rows are zero
    assert np.array_equal(unpad.gather_rows(back, idx), g)
    # sequence i of the packed tensor is rows cu[i] .. cu[i+1]-1, in position order
    for i in range(5):
        assert np.array_equal(g[cu[i]:cu[i + 1]], x[6 * i:6 * i + (cu[i + 1] - cu[i])])
