"""Pins for oracle/layernorm.py: closed forms, invariants, torch's own layer_norm and
autograd (CPU, fp64) as an independent implementation, finite differences, and the mask's
element-to-byte map looked up by hand.  No GPU."""
import numpy as np
import pytest
import torch

from oracle import dropout_mask as dm
from oracle import layernorm as ln

RNG = np.random.default_rng(173)


def data(t, n):
    return (RNG.standard_normal((t, n)), RNG.standard_normal((t, n)), 1.0 + 0.3 * RNG.standard_normal(n),
            RNG.standard_normal(n), RNG.standard_normal((t, n)))


def test_closed_forms():
    x, r, gamma, beta, _ = data(5, 32)
    y, z, mu, rstd = ln.fwd(x, r, np.ones(32), np.zeros(32), 0.0)
    assert np.allclose(z, x + r) and np.abs(y.mean(axis=1)).max() < 1e-14
    assert np.abs((y ** 2).mean(axis=1) - 1.0).max() < 1e-12
    # a constant row has zero variance: y = beta exactly, rstd = eps^-1/2
    y, _, mu, rstd = ln.fwd(np.full((1, 32), 2.5), np.full((1, 32), 0.5), gamma, beta, 1e-5)
    assert np.array_equal(y[0], beta) and mu[0] == 3.0 and abs(rstd[0] - 1e-5 ** -0.5) < 1e-9
    # hand-worked: z = [1, 3], mu = 2, var = 1, eps = 3 -> rstd = 1/2, xh = [-1/2, 1/2]
    y, _, mu, rstd = ln.fwd(np.array([[1.0, 1.0]]), np.array([[0.0, 2.0]]), np.array([2.0, 4.0]), np.array([1.0, -1.0]), 3.0)
    assert mu[0] == 2.0 and rstd[0] == 0.5 and y[0].tolist() == [0.0, 1.0]


@pytest.mark.parametrize("p", [0.0, 0.3])
def test_against_torch_layer_norm_and_autograd(p):
    t, n, eps = 7, 48, 1e-5
    x, r, gamma, beta, dy = data(t, n)
    mask = ln.ln_keep_mask(t, n, p, 9) if p else None
    c = dm.keep_scale(p)
    y, z, mu, rstd = ln.fwd(x, r, gamma, beta, eps, mask, c)
    dx, dr, dgamma, dbeta = ln.bwd(dy, x, r, gamma, eps, mask, c)
    tx, tr, tg, tb = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, r, gamma, beta))
    tz = tx * (torch.tensor(mask * c, dtype=torch.float64) if p else 1.0) + tr
    ty = torch.nn.functional.layer_norm(tz, (n,), tg, tb, eps)
    ty.backward(torch.tensor(dy))
    assert np.abs(y - ty.detach().numpy()).max() < 1e-12
    for got, want in ((dx, tx.grad), (dr, tr.grad), (dgamma, tg.grad), (dbeta, tb.grad)):
        assert np.abs(got - want.numpy()).max() < 1e-11


def test_invariants():
    t, n, eps = 4, 64, 1e-5
    x, r, gamma, beta, dy = data(t, n)
    y, *_ = ln.fwd(x, r, gamma, beta, eps)
    y2, *_ = ln.fwd(x + 3.7, r, gamma, beta, eps)               # shift invariance
    assert np.abs(y - y2).max() < 1e-12
    dx, dr, dgamma, dbeta = ln.bwd(dy, x, r, gamma, eps)
    assert np.abs(dr.sum(axis=1)).max() < 1e-12                  # dz is orthogonal to the constant vector
    assert np.array_equal(dx, dr)                                # no dropout: same gradient to both inputs
    assert np.allclose(dbeta, dy.sum(axis=0))
    mask = ln.ln_keep_mask(t, n, 0.5, 3)
    dx, dr, *_ = ln.bwd(dy, x, r, gamma, eps, mask, 2.0)
    assert np.array_equal(dx, dr * mask * 2.0)
    assert (dx[mask == 0] == 0).all()


def test_finite_differences_with_dropout():
    t, n, eps = 3, 16, 1e-3
    x, r, gamma, beta, dy = data(t, n)
    mask = ln.ln_keep_mask(t, n, 0.25, 5)
    c = dm.keep_scale(0.25)
    loss = lambda x_, r_, g_, b_: float((ln.fwd(x_, r_, g_, b_, eps, mask, c)[0] * dy).sum())
    grads = ln.bwd(dy, x, r, gamma, eps, mask, c)
    args = [x, r, gamma, beta]
    h = 1e-6
    for which in range(4):
        for _ in range(4):
            d = RNG.standard_normal(args[which].shape)
            ap, am = list(args), list(args)
            ap[which] = args[which] + h * d
            am[which] = args[which] - h * d
            fd = (loss(*ap) - loss(*am)) / (2 * h)
            an = float((grads[which] * d).sum())
            assert abs(fd - an) <= 1e-7 * max(1.0, abs(an))


def test_mask_bytes_looked_up_by_hand():
    seed, t = 0xABCDEF0123456789, 6
    m = ln.ln_keep_mask(8, 64, 0.5, seed)
    key = (seed & 0xFFFFFFFF, seed >> 32)
    # column 37 of row 6: call (37 >> 4 = 2, 6, tag, 0), byte 37 & 15 = 5 -> word 1, byte 1
    out = dm.philox4x32_10(np.array([[2, t, ln.LN_TAG, 0]], dtype=np.uint32), key)[0]
    assert m[t, 37] == (((int(out[1]) >> 8) & 0xFF) >= 128)
    # column 15 of row 0: call (0, 0, tag, 0), word 3, byte 3
    out = dm.philox4x32_10(np.array([[0, 0, ln.LN_TAG, 0]], dtype=np.uint32), key)[0]
    assert m[0, 15] == (((int(out[3]) >> 24) & 0xFF) >= 128)
    assert np.array_equal(ln.ln_keep_mask(3, 64, 0.5, seed, first_row=5), m[5:8])
    big = ln.ln_keep_mask(300, 1024, 0.1, 1)
    pk = 1 - 26 / 256
    assert abs(big.mean() - pk) < 5 * np.sqrt(pk * (1 - pk) / big.size)
