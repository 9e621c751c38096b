"""Pins for the fp64 CPU oracle: everything here checks oracle/ against
something other than itself -- hand-worked values, closed forms, invariants of
softmax attention, an independent brute force, finite differences, and a
library softmax.  No GPU, no HIP library."""
import math
import os

import numpy as np
import pytest

from oracle import oracle

RNG = np.random.default_rng(20220808)


def rand(*shape):
    return RNG.standard_normal(shape)


def cu_of(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


# --------------------------------------------------------------------------
# independent brute force: pure Python scalars, no max subtraction, explicit
# normalisation, and the gradient through the full softmax Jacobian
# (dS_rj = sum_k dP_rk * P_rk * (delta_jk - P_rj)) rather than the compact
# P o (dP - D) form the oracle uses.
# --------------------------------------------------------------------------
def brute_fwd(q, k, v, lengths, scale):
    t, h, d = q.shape
    o = [[[0.0] * d for _ in range(h)] for _ in range(t)]
    lse = [[0.0] * t for _ in range(h)]
    r0 = 0
    for L in lengths:
        for hh in range(h):
            for r in range(r0, r0 + L):
                e = []
                for j in range(r0, r0 + L):
                    s = 0.0
                    for c in range(d):
                        s += float(q[r, hh, c]) * float(k[j, hh, c])
                    e.append(math.exp(s * scale))
                z = sum(e)
                lse[hh][r] = math.log(z)
                for c in range(d):
                    acc = 0.0
                    for jj, j in enumerate(range(r0, r0 + L)):
                        acc += e[jj] / z * float(v[j, hh, c])
                    o[r][hh][c] = acc
        r0 += L
    return np.array(o).reshape(t, h, d), np.array(lse).reshape(h, t)


def brute_bwd(q, k, v, do, lengths, scale):
    t, h, d = q.shape
    dq, dk, dv = np.zeros((t, h, d)), np.zeros((t, h, d)), np.zeros((t, h, d))
    r0 = 0
    for L in lengths:
        for hh in range(h):
            for r in range(r0, r0 + L):
                e = [math.exp(scale * sum(float(q[r, hh, c]) * float(k[j, hh, c]) for c in range(d)))
                     for j in range(r0, r0 + L)]
                z = sum(e)
                p = [x / z for x in e]
                dp = [sum(float(do[r, hh, c]) * float(v[j, hh, c]) for c in range(d))
                      for j in range(r0, r0 + L)]
                for jj in range(L):
                    ds = 0.0
                    for kk in range(L):
                        ds += dp[kk] * p[kk] * ((1.0 if kk == jj else 0.0) - p[jj])
                    for c in range(d):
                        dq[r, hh, c] += scale * ds * float(k[r0 + jj, hh, c])
                        dk[r0 + jj, hh, c] += scale * ds * float(q[r, hh, c])
                        dv[r0 + jj, hh, c] += 0.0
                for jj in range(L):
                    for c in range(d):
                        dv[r0 + jj, hh, c] += p[jj] * float(do[r, hh, c])
        r0 += L
    return dq, dk, dv


@pytest.mark.parametrize("lengths,h,d", [([1], 1, 2), ([2, 3], 2, 3), ([6, 1, 4], 2, 4),
                                         ([3, 5], 2, 64), ([0, 4, 0, 2], 1, 8)])
def test_brute_force_tiny(lengths, h, d):
    t = sum(lengths)
    q, k, v, do = rand(t, h, d), rand(t, h, d), rand(t, h, d), rand(t, h, d)
    scale = 1.0 / math.sqrt(d)
    o, lse = oracle.fwd(q, k, v, cu_of(lengths), scale)
    bo, blse = brute_fwd(q, k, v, lengths, scale)
    np.testing.assert_allclose(o, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, blse, rtol=0, atol=1e-13)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu_of(lengths), scale)
    bq, bk, bv = brute_bwd(q, k, v, do, lengths, scale)
    np.testing.assert_allclose(dq, bq, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dk, bk, rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, bv, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------
# hand-worked example (tests/golden/two_key_example.txt)
# --------------------------------------------------------------------------
def read_golden(name):
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    out = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        f = line.split()
        out[f[0]] = np.array([float(x) for x in f[3:]]).reshape(int(f[1]), int(f[2]))
    return out


def test_hand_worked_two_keys():
    g = read_golden("two_key_example.txt")
    q = np.array([[1.0, 0.0], [0.0, 0.0]]).reshape(2, 1, 2)
    k = np.array([[0.0, 0.0], [math.log(3.0), 0.0]]).reshape(2, 1, 2)
    v = np.array([[4.0, 0.0], [0.0, 8.0]]).reshape(2, 1, 2)
    do = np.array([[1.0, 1.0], [0.0, 0.0]]).reshape(2, 1, 2)
    cu = cu_of([2])
    o, lse = oracle.fwd(q, k, v, cu, 1.0)
    np.testing.assert_allclose(o.reshape(2, 2), g["O"], atol=1e-15)
    np.testing.assert_allclose(lse, g["LSE"], atol=1e-15)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, 1.0)
    np.testing.assert_allclose(dq.reshape(2, 2), g["dQ"], atol=1e-15)
    np.testing.assert_allclose(dk.reshape(2, 2), g["dK"], atol=1e-15)
    np.testing.assert_allclose(dv.reshape(2, 2), g["dV"], atol=1e-15)


# --------------------------------------------------------------------------
# closed forms
# --------------------------------------------------------------------------
def test_length_one_returns_v():
    lengths = [1, 1, 1]
    q, k, v, do = (rand(3, 2, 64) for _ in range(4))
    o, lse = oracle.fwd(q, k, v, cu_of(lengths), 0.125)
    np.testing.assert_array_equal(o, v)
    np.testing.assert_allclose(lse.T, 0.125 * (q * k).sum(-1), atol=1e-14)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu_of(lengths), 0.125)
    np.testing.assert_array_equal(dv, do)
    assert np.abs(dq).max() == 0 and np.abs(dk).max() == 0


def test_zero_scale_is_uniform_average():
    lengths = [5, 9]
    t = sum(lengths)
    q, k, v, do = (rand(t, 2, 64) for _ in range(4))
    cu = cu_of(lengths)
    o, lse = oracle.fwd(q, k, v, cu, 0.0)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, 0.0)
    for i, L in enumerate(lengths):
        sl = slice(cu[i], cu[i + 1])
        np.testing.assert_allclose(o[sl], np.broadcast_to(v[sl].mean(0), o[sl].shape), atol=1e-14)
        np.testing.assert_allclose(lse[:, sl], math.log(L), atol=1e-14)
        np.testing.assert_allclose(dv[sl], np.broadcast_to(do[sl].sum(0) / L, dv[sl].shape), atol=1e-14)
    assert np.abs(dq).max() == 0 and np.abs(dk).max() == 0


def test_zero_query_gives_mean_and_no_dk():
    lengths = [7]
    q = np.zeros((7, 1, 64))
    k, v, do = rand(7, 1, 64), rand(7, 1, 64), rand(7, 1, 64)
    o, lse = oracle.fwd(q, k, v, cu_of(lengths), 0.125)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(0), o.shape), atol=1e-14)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu_of(lengths), 0.125)
    assert np.abs(dk).max() == 0
    # dQ_r = scale * sum_j (1/L) (dP_rj - mean_j dP_rj) K_j: in general non-zero
    dp = do[:, 0] @ v[:, 0].T
    ds = (dp - dp.mean(1, keepdims=True)) / 7
    np.testing.assert_allclose(dq[:, 0], 0.125 * ds @ k[:, 0], atol=1e-13)


def test_constant_v_gives_constant_output_and_rows_sum_to_one():
    lengths = [4, 33, 130]
    t = sum(lengths)
    q, k, do = rand(t, 2, 64), rand(t, 2, 64), rand(t, 2, 64)
    vrow = rand(1, 2, 64)
    v = np.broadcast_to(vrow, (t, 2, 64)).copy()
    o, _ = oracle.fwd(q, k, v, cu_of(lengths), 0.125)
    np.testing.assert_allclose(o, v, atol=1e-14)
    # V = 1 reads the softmax row sums directly
    o1, _ = oracle.fwd(q, k, np.ones((t, 2, 64)), cu_of(lengths), 0.125)
    np.testing.assert_allclose(o1, 1.0, atol=1e-14)
    dq, dk, _ = oracle.bwd(q, k, v, do, cu_of(lengths), 0.125)
    assert np.abs(dq).max() < 1e-13 and np.abs(dk).max() < 1e-13


def test_one_hot_limit_picks_the_value_row():
    L = 6
    k = np.zeros((L, 1, 64))
    k[2, 0, 0] = 1000.0
    q = np.zeros((L, 1, 64))
    q[:, 0, 0] = 1.0
    v = rand(L, 1, 64)
    o, lse = oracle.fwd(q, k, v, cu_of([L]), 1.0)
    np.testing.assert_allclose(o, np.broadcast_to(v[2], o.shape), atol=1e-12)
    np.testing.assert_allclose(lse, 1000.0, atol=1e-9)


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
def test_shift_of_keys_leaves_output_unchanged():
    lengths = [9, 20]
    t = sum(lengths)
    q, k, v = rand(t, 2, 64), rand(t, 2, 64), rand(t, 2, 64)
    o, lse = oracle.fwd(q, k, v, cu_of(lengths), 0.125)
    shift = rand(1, 2, 64)
    o2, lse2 = oracle.fwd(q, k + shift, v, cu_of(lengths), 0.125)
    np.testing.assert_allclose(o2, o, atol=1e-12)
    # LSE moves by the per-row constant scale * q.c
    np.testing.assert_allclose(lse2 - lse, (0.125 * (q * shift).sum(-1)).T, atol=1e-12)


def test_key_and_query_permutations():
    L = 11
    q, k, v, do = (rand(L, 2, 64) for _ in range(4))
    cu = cu_of([L])
    o, lse = oracle.fwd(q, k, v, cu, 0.125)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, 0.125)
    perm = RNG.permutation(L)
    o2, _ = oracle.fwd(q, k[perm], v[perm], cu, 0.125)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    dq2, dk2, dv2 = oracle.bwd(q, k[perm], v[perm], do, cu, 0.125)
    np.testing.assert_allclose(dq2, dq, atol=1e-13)
    np.testing.assert_allclose(dk2, dk[perm], atol=1e-13)
    np.testing.assert_allclose(dv2, dv[perm], atol=1e-13)
    o3, lse3 = oracle.fwd(q[perm], k, v, cu, 0.125)
    np.testing.assert_allclose(o3, o[perm], atol=1e-13)
    np.testing.assert_allclose(lse3, lse[:, perm], atol=1e-13)


def test_gradient_sum_rules():
    lengths = [13, 2, 40]
    t = sum(lengths)
    q, k, v, do = (rand(t, 3, 64) for _ in range(4))
    cu = cu_of(lengths)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, 0.125)
    for i in range(len(lengths)):
        sl = slice(cu[i], cu[i + 1])
        np.testing.assert_allclose(dv[sl].sum(0), do[sl].sum(0), atol=1e-12)  # P rows sum to 1
        np.testing.assert_allclose(dk[sl].sum(0), 0.0, atol=1e-12)            # dS rows sum to 0


def test_sequences_and_heads_are_independent_and_pack_order_is_free():
    lengths = [5, 12, 3]
    t = sum(lengths)
    q, k, v, do = (rand(t, 2, 64) for _ in range(4))
    cu = cu_of(lengths)
    o, lse = oracle.fwd(q, k, v, cu, 0.125)
    g = oracle.bwd(q, k, v, do, cu, 0.125)
    # perturb sequence 1 and head 1: sequence 0/2 and head 0 must not move
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    for a in (q2, k2, v2):
        a[cu[1]:cu[2]] += 1.0
        a[:, 1] *= 2.0
    o2, _ = oracle.fwd(q2, k2, v2, cu, 0.125)
    g2 = oracle.bwd(q2, k2, v2, do, cu, 0.125)
    keep = np.r_[0:cu[1], cu[2]:cu[3]]
    np.testing.assert_array_equal(o2[keep, 0], o[keep, 0])
    for a, b in zip(g, g2):
        np.testing.assert_array_equal(b[keep, 0], a[keep, 0])
    # each sequence alone, and the pack in another order
    for i in range(3):
        sl = slice(cu[i], cu[i + 1])
        oi, lsei = oracle.fwd(q[sl], k[sl], v[sl], cu_of([lengths[i]]), 0.125)
        np.testing.assert_array_equal(oi, o[sl])
        np.testing.assert_array_equal(lsei, lse[:, sl])
        gi = oracle.bwd(q[sl], k[sl], v[sl], do[sl], cu_of([lengths[i]]), 0.125)
        for a, b in zip(g, gi):
            np.testing.assert_array_equal(b, a[sl])
    order = [2, 0, 1]
    idx = np.concatenate([np.arange(cu[i], cu[i + 1]) for i in order])
    o3, _ = oracle.fwd(q[idx], k[idx], v[idx], cu_of([lengths[i] for i in order]), 0.125)
    np.testing.assert_array_equal(o3, o[idx])


def test_padded_with_mask_equals_unpadded():
    lengths = np.array([5, 16, 1, 9])
    t, m = int(lengths.sum()), 16
    q, k, v, do = (rand(t, 2, 64) for _ in range(4))
    cu = cu_of(lengths)
    o, lse = oracle.fwd(q, k, v, cu, 0.125)
    g = oracle.bwd(q, k, v, do, cu, 0.125)
    # padded layout, pad rows hold garbage (finite) values
    pad = {}
    rows = np.concatenate([i * m + np.arange(L) for i, L in enumerate(lengths)])
    for name, x in (("q", q), ("k", k), ("v", v)):
        p = rand(len(lengths) * m, 2, 64) * 10
        p[rows] = x
        pad[name] = p
    pdo = np.zeros((len(lengths) * m, 2, 64))   # loss ignores the pad rows
    pdo[rows] = do
    cup = (np.arange(len(lengths) + 1) * m).astype(np.int32)
    op, lsep = oracle.fwd(pad["q"], pad["k"], pad["v"], cup, 0.125, seqused=lengths)
    np.testing.assert_allclose(op[rows], o, atol=1e-14)
    np.testing.assert_allclose(lsep[:, rows], lse, atol=1e-14)
    gp = oracle.bwd(pad["q"], pad["k"], pad["v"], pdo, cup, 0.125, seqused=lengths)
    for a, b in zip(g, gp):
        np.testing.assert_allclose(b[rows], a, atol=1e-13)
    # masked keys receive no gradient
    mask = np.ones(len(lengths) * m, bool)
    mask[rows] = False
    assert np.abs(gp[1][mask]).max() == 0 and np.abs(gp[2][mask]).max() == 0


def test_seqused_zero_row_convention():
    q, k, v, do = (rand(4, 1, 8) for _ in range(4))
    o, lse = oracle.fwd(q, k, v, cu_of([4]), 0.3, seqused=[0])
    assert np.abs(o).max() == 0 and np.all(np.isneginf(lse))
    for g in oracle.bwd(q, k, v, do, cu_of([4]), 0.3, seqused=[0]):
        assert np.abs(g).max() == 0


def test_seqused_is_clamped_to_the_sequence():
    """A key count beyond the sequence means "all keys", a negative one "none": the count
    describes padding, it never makes the oracle read another sequence's rows (the two
    sequences here would otherwise see each other)."""
    q, k, v, do = (rand(9, 2, 8) for _ in range(4))
    cu = cu_of([4, 5])
    full = oracle.fwd(q, k, v, cu, 0.3), oracle.bwd(q, k, v, do, cu, 0.3)
    over = oracle.fwd(q, k, v, cu, 0.3, seqused=[7, 500]), oracle.bwd(q, k, v, do, cu, 0.3, seqused=[7, 500])
    for a, b in zip(full[0] + full[1], over[0] + over[1]):
        assert np.array_equal(a, b)
    none = oracle.fwd(q, k, v, cu, 0.3, seqused=[-1, 5])
    assert np.abs(none[0][:4]).max() == 0 and np.all(np.isneginf(none[1][:, :4]))
    assert np.array_equal(none[0][4:], full[0][0][4:])


# --------------------------------------------------------------------------
# library special case: scipy's softmax + numpy matmul per (sequence, head)
# --------------------------------------------------------------------------
def test_against_scipy_softmax():
    scipy_special = pytest.importorskip("scipy.special")
    lengths = [17, 64, 3, 128]
    t = sum(lengths)
    q, k, v = rand(t, 2, 64), rand(t, 2, 64), rand(t, 2, 64)
    cu = cu_of(lengths)
    o, lse = oracle.fwd(q, k, v, cu, 0.125)
    for i in range(len(lengths)):
        sl = slice(cu[i], cu[i + 1])
        for h in range(2):
            s = 0.125 * q[sl, h] @ k[sl, h].T
            np.testing.assert_allclose(o[sl, h], scipy_special.softmax(s, axis=1) @ v[sl, h],
                                       atol=1e-13)
            np.testing.assert_allclose(lse[h, sl], scipy_special.logsumexp(s, axis=1), atol=1e-13)


# --------------------------------------------------------------------------
# finite differences of  loss = sum(O o dO)
# --------------------------------------------------------------------------
def test_gradients_against_central_differences():
    lengths = [6, 1, 19]
    t = sum(lengths)
    q, k, v, do = (rand(t, 2, 64) for _ in range(4))
    cu = cu_of(lengths)
    dq, dk, dv = oracle.bwd(q, k, v, do, cu, 0.125)

    def loss(qq, kk, vv):
        return float((oracle.fwd(qq, kk, vv, cu, 0.125)[0] * do).sum())

    eps = 1e-5
    # random directions
    for _ in range(4):
        uq, uk, uv = rand(*q.shape), rand(*q.shape), rand(*q.shape)
        fd = (loss(q + eps * uq, k + eps * uk, v + eps * uv)
              - loss(q - eps * uq, k - eps * uk, v - eps * uv)) / (2 * eps)
        an = float((dq * uq).sum() + (dk * uk).sum() + (dv * uv).sum())
        assert abs(fd - an) <= 1e-7 * max(1.0, abs(an))
    # single coordinates of each tensor separately
    for which, grad in (("q", dq), ("k", dk), ("v", dv)):
        for _ in range(6):
            idx = (RNG.integers(t), RNG.integers(2), RNG.integers(64))
            e = np.zeros_like(q)
            e[idx] = eps
            args_p = {"q": q, "k": k, "v": v}
            args_m = dict(args_p)
            args_p[which] = args_p[which] + e
            args_m[which] = args_m[which] - e
            fd = (loss(args_p["q"], args_p["k"], args_p["v"])
                  - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
            assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), (which, idx)


def test_bad_prefix_sums_are_rejected():
    q = rand(4, 1, 8)
    with pytest.raises((ValueError, AssertionError)):
        oracle.fwd(q, q, q, np.array([0, 3, 2, 4], dtype=np.int32), 1.0)
    with pytest.raises((ValueError, AssertionError)):
        oracle.fwd(q, q, q, np.array([1, 4], dtype=np.int32), 1.0)
