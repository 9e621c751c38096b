"""Pins for oracle/embedding.py: hand-worked case, closed forms, numpy's add.at and torch's
embedding autograd (fp64) as independent implementations, order invariance.  No GPU."""
import numpy as np
import torch

from oracle import embedding as emb

RNG = np.random.default_rng(174)


def test_hand_worked():
    dy = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0], [5.0, 5.0]])
    dw, cnt = emb.embedding_bwd(dy, [2, 0, 2, 7], vocab=3)
    assert dw.tolist() == [[10.0, 20.0], [0.0, 0.0], [101.0, 202.0]] and cnt.tolist() == [1, 0, 2]
    dw, cnt = emb.embedding_bwd(dy, [2, 0, 2, 1], vocab=3, padding_idx=2)
    assert dw.tolist() == [[10.0, 20.0], [5.0, 5.0], [0.0, 0.0]]


def test_closed_forms_and_library_routines():
    t, n, v = 500, 24, 37
    dy = RNG.standard_normal((t, n))
    idx = RNG.integers(0, v, size=t)
    dw, cnt = emb.embedding_bwd(dy, idx, v)
    ref = np.zeros((v, n))
    np.add.at(ref, idx, dy)
    assert np.abs(dw - ref).max() < 1e-12 and np.array_equal(cnt, np.bincount(idx, minlength=v))
    same, _ = emb.embedding_bwd(dy, np.full(t, 5), v)
    assert np.abs(same[5] - dy.sum(axis=0)).max() < 1e-12 and (np.delete(same, 5, axis=0) == 0).all()
    perm = RNG.permutation(t)
    dw2, _ = emb.embedding_bwd(dy[perm], idx[perm], v)
    assert np.abs(dw2 - dw).max() < 1e-12                       # the order of the tokens does not matter
    w = torch.zeros((v, n), dtype=torch.float64, requires_grad=True)
    out = torch.nn.functional.embedding(torch.from_numpy(idx), w, padding_idx=3)
    out.backward(torch.from_numpy(dy))
    dw3, _ = emb.embedding_bwd(dy, idx, v, padding_idx=3)
    assert np.abs(dw3 - w.grad.numpy()).max() < 1e-12
    init = RNG.standard_normal((v, n))
    dw4, _ = emb.embedding_bwd(dy, idx, v, dw_init=init)
    assert np.abs(dw4 - (init + dw)).max() < 1e-12
    a = emb.abs_sums(dy, idx, v)
    assert (a >= np.abs(dw) - 1e-12).all()
