"""Pins for the dropout side of the CPU oracle: the counter-based generator
against its published known-answer vectors, the keep mask's structure against
its definition, and the masked attention against brute force, closed forms,
invariants and finite differences.  No GPU, no HIP library."""
import math
import os

import numpy as np
import pytest

from oracle import dropout_mask as dm
from oracle import oracle

RNG = np.random.default_rng(20220809)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def cu_of(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def rand(*shape):
    return RNG.standard_normal(shape)


# ------------------------------------------------------------------ generator
def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(x, 16) for x in r]
        out = dm.philox4x32_10(np.array([w[0:4]], dtype=np.uint32), (w[4], w[5]))[0]
        assert [int(x) for x in out] == w[6:10]


def test_philox_is_elementwise_over_a_batch():
    ctr = RNG.integers(0, 2 ** 32, size=(5, 7, 4), dtype=np.uint64).astype(np.uint32)
    out = dm.philox4x32_10(ctr, (123, 456))
    for i in (0, 4):
        for j in (0, 6):
            assert np.array_equal(out[i, j], dm.philox4x32_10(ctr[i, j][None], (123, 456))[0])


# ----------------------------------------------------------------------- mask
def test_threshold_quantisation():
    assert dm.threshold(0.0) == 0 and dm.keep_scale(0.0) == 1.0
    assert dm.threshold(0.1) == 26 and dm.keep_scale(0.1) == 256.0 / 230.0
    assert dm.threshold(0.5) == 128 and dm.keep_scale(0.5) == 2.0
    assert dm.threshold(0.999) == 255
    with pytest.raises(ValueError):
        dm.threshold(1.0)
    with pytest.raises(ValueError):
        dm.threshold(-0.1)


def test_every_block_uses_each_byte_of_its_call_once():
    """Within a 4x4 block the 16 elements map one-to-one onto the 16 output bytes of
    the call with counter (K4, Q4, r0, head) and key = the seed's two halves."""
    seed, r0, heads = 0x1234567890ABCDEF, 37, 3
    by = dm.random_bytes(r0, heads, 24, 40, seed)
    key = (seed & 0xFFFFFFFF, seed >> 32)
    for h in range(heads):
        for q4 in range(6):
            for k4 in range(10):
                out = dm.philox4x32_10(np.array([[k4, q4, r0, h]], dtype=np.uint32), key)[0]
                call_bytes = sorted(int((w >> (8 * y)) & 0xFF) for w in out for y in range(4))
                blk = by[h, 4 * q4:4 * q4 + 4, 4 * k4:4 * k4 + 4]
                assert sorted(int(x) for x in blk.ravel()) == call_bytes


def test_element_to_byte_map_written_out():
    """Two elements looked up by hand: (q, k) = (5, 9) and (14, 3)."""
    seed, r0 = 99, 0
    by = dm.random_bytes(r0, 1, 16, 16, seed)
    key = (99, 0)
    # q = 5, k = 9: block (1, 2); x = ((5&3) - (9>>3)) & 3 = 0; y = ((9&3) - (5>>3)) & 3 = 1
    out = dm.philox4x32_10(np.array([[2, 1, 0, 0]], dtype=np.uint32), key)[0]
    assert by[0, 5, 9] == (int(out[0]) >> 8) & 0xFF
    # q = 14, k = 3: block (3, 0); x = ((14&3) - 0) & 3 = 2; y = (3 - 1) & 3 = 2
    out = dm.philox4x32_10(np.array([[0, 3, 0, 0]], dtype=np.uint32), key)[0]
    assert by[0, 14, 3] == (int(out[2]) >> 16) & 0xFF


def test_mask_depends_on_seed_head_and_sequence_start():
    a = dm.random_bytes(0, 2, 32, 32, 7)
    assert not np.array_equal(a[0], a[1])                                   # head
    assert not np.array_equal(a, dm.random_bytes(0, 2, 32, 32, 8))          # seed
    assert not np.array_equal(a, dm.random_bytes(0, 2, 32, 32, 7 + 2 ** 32))  # high half of the seed
    assert not np.array_equal(a, dm.random_bytes(32, 2, 32, 32, 7))         # start row
    # the mask of a sequence does not depend on what else is in the pack
    m1 = dm.keep_masks(cu_of([5, 9]), 2, 0.3, 7)
    m2 = dm.keep_masks(cu_of([5, 9, 4]), 2, 0.3, 7)
    assert np.array_equal(m1[1], m2[1])
    # a longer sequence at the same start extends the shorter one's mask
    m3 = dm.keep_masks(cu_of([5, 12]), 2, 0.3, 7)
    assert np.array_equal(m3[1][:, :9, :9], m1[1])


@pytest.mark.parametrize("p", [0.0, 0.1, 0.5, 0.9])
def test_kept_fraction(p):
    masks = dm.keep_masks(cu_of([200, 57]), 4, p, 2024)
    n = sum(m.size for m in masks)
    kept = sum(int(m.sum()) for m in masks)
    pk = 1.0 - dm.threshold(p) / 256.0
    assert abs(kept - n * pk) <= 5.0 * math.sqrt(n * pk * (1 - pk)) + 1e-9
    if p == 0.0:
        assert kept == n
    # rows and columns are not degenerate either
    m = masks[0][0].astype(np.float64)
    if 0 < p < 1:
        assert m.mean(axis=0).std() < 0.1 and m.mean(axis=1).std() < 0.1


# --------------------------------------------------------- masked attention
def dense_masked(q, k, v, do, lengths, scale, masks, c):
    """Independent formulation per (sequence, head) with dense fp64 numpy: explicit
    normalisation without max subtraction, gradient through the full softmax Jacobian."""
    t, h, d = q.shape
    o, dq, dk, dv = (np.zeros((t, h, d)) for _ in range(4))
    lse = np.zeros((h, t))
    r0 = 0
    for i, n in enumerate(lengths):
        sl = slice(r0, r0 + n)
        for hh in range(h):
            e = np.exp(scale * q[sl, hh] @ k[sl, hh].T)
            z = e.sum(axis=1, keepdims=True)
            p = e / z
            w = p * masks[i][hh] * c
            o[sl, hh] = w @ v[sl, hh]
            lse[hh, sl] = np.log(z[:, 0])
            if do is not None:
                g = do[sl, hh]
                dv[sl, hh] = w.T @ g
                dw = g @ v[sl, hh].T                 # gradient w.r.t. the dropped probabilities
                dp = dw * masks[i][hh] * c           # ... w.r.t. the softmax output
                ds = np.zeros_like(p)
                for r in range(n):                   # full Jacobian of one softmax row
                    jac = np.diag(p[r]) - np.outer(p[r], p[r])
                    ds[r] = jac @ dp[r]
                dq[sl, hh] = scale * ds @ k[sl, hh]
                dk[sl, hh] = scale * ds.T @ q[sl, hh]
        r0 += n
    return o, lse, dq, dk, dv


def make(lengths, h, d=8):
    t = int(sum(lengths))
    return rand(t, h, d), rand(t, h, d), rand(t, h, d), rand(t, h, d)


def test_masked_attention_against_dense_formulation():
    lengths, h, scale = [1, 6, 13], 2, 0.4
    q, k, v, do = make(lengths, h)
    cu = cu_of(lengths)
    masks = dm.keep_masks(cu, h, 0.35, 5)
    c = dm.keep_scale(0.35)
    o, lse = oracle.fwd_dropout(q, k, v, cu, scale, masks, c)
    dq, dk, dv = oracle.bwd_dropout(q, k, v, do, cu, scale, masks, c)
    ro, rlse, rdq, rdk, rdv = dense_masked(q, k, v, do, lengths, scale, masks, c)
    for a, b in ((o, ro), (lse, rlse), (dq, rdq), (dk, rdk), (dv, rdv)):
        assert np.max(np.abs(a - b)) < 1e-12


def test_all_kept_is_plain_attention():
    lengths, h = [4, 9], 2
    q, k, v, do = make(lengths, h)
    cu = cu_of(lengths)
    masks = [np.ones((h, n, n), dtype=np.uint8) for n in lengths]
    o, lse = oracle.fwd_dropout(q, k, v, cu, 0.3, masks, 1.0)
    o0, lse0 = oracle.fwd(q, k, v, cu, 0.3)
    assert np.array_equal(o, o0) and np.array_equal(lse, lse0)
    g = oracle.bwd_dropout(q, k, v, do, cu, 0.3, masks, 1.0)
    g0 = oracle.bwd(q, k, v, do, cu, 0.3)
    for a, b in zip(g, g0):
        assert np.array_equal(a, b)


def test_dropping_a_key_everywhere_zeroes_its_value_but_not_the_normaliser():
    """Mask applied AFTER the softmax: dropping key j in every row equals attention with
    V_j = 0 (times c); the row sums, hence LSE, still include key j."""
    lengths, h, j, c = [7], 1, 3, 1.6
    q, k, v, do = make(lengths, h)
    cu = cu_of(lengths)
    m = np.ones((h, 7, 7), dtype=np.uint8)
    m[:, :, j] = 0
    o, lse = oracle.fwd_dropout(q, k, v, cu, 0.5, [m], c)
    v0 = v.copy()
    v0[j] = 0.0
    o0, lse0 = oracle.fwd(q, k, v0, cu, 0.5)
    assert np.max(np.abs(o - c * o0)) < 1e-13
    assert np.array_equal(lse, lse0)
    dq, dk, dv = oracle.bwd_dropout(q, k, v, do, cu, 0.5, [m], c)
    assert np.all(dv[j] == 0.0)


def test_invariants_under_dropout():
    lengths, h, scale = [10, 5], 2, 0.25
    q, k, v, do = make(lengths, h)
    cu = cu_of(lengths)
    masks = dm.keep_masks(cu, h, 0.5, 11)
    o1, _ = oracle.fwd_dropout(q, k, v, cu, scale, masks, 1.0)
    o2, _ = oracle.fwd_dropout(q, k, v, cu, scale, masks, 2.0)
    assert np.max(np.abs(o2 - 2.0 * o1)) < 1e-14                   # linear in c
    dq, dk, dv = oracle.bwd_dropout(q, k, v, do, cu, scale, masks, 2.0)
    for i in range(len(lengths)):                                   # rows of dS sum to zero
        assert np.max(np.abs(dk[cu[i]:cu[i + 1]].sum(axis=0))) < 1e-12
    # adding a constant vector to every key of a sequence changes nothing (softmax shift)
    k2 = k + rand(1, h, k.shape[2])
    o3, _ = oracle.fwd_dropout(q, k2, v, cu, scale, masks, 2.0)
    assert np.max(np.abs(o3 - o2)) < 1e-12


def test_finite_differences_with_a_fixed_mask():
    lengths, h, scale = [3, 8], 2, 0.35
    q, k, v, do = make(lengths, h, d=4)
    cu = cu_of(lengths)
    masks = dm.keep_masks(cu, h, 0.4, 3)
    c = dm.keep_scale(0.4)

    def loss(q_, k_, v_):
        o, _ = oracle.fwd_dropout(q_, k_, v_, cu, scale, masks, c)
        return float((o * do).sum())

    grads = oracle.bwd_dropout(q, k, v, do, cu, scale, masks, c)
    eps = 1e-6
    for which, g in enumerate(grads):
        for _ in range(6):
            dirn = rand(*q.shape)
            args_p = [q, k, v]
            args_m = [q, k, v]
            args_p[which] = args_p[which] + eps * dirn
            args_m[which] = args_m[which] - eps * dirn
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            an = float((g * dirn).sum())
            assert abs(fd - an) <= 1e-7 * max(1.0, abs(an))


def test_seqused_with_dropout():
    """Keys at or beyond seqused stay excluded; the mask is indexed by true positions."""
    lengths, h = [9], 1
    q, k, v, do = make(lengths, h)
    cu = cu_of(lengths)
    masks = dm.keep_masks(cu, h, 0.3, 21)
    c = dm.keep_scale(0.3)
    su = np.array([5], dtype=np.int32)
    o, lse = oracle.fwd_dropout(q, k, v, cu, 0.5, masks, c, seqused=su)
    # the same as a 9-row sequence whose keys 5.. are pushed to -inf: emulate with explicit softmax
    e = np.exp(0.5 * q[:, 0] @ k[:5, 0].T)
    p = e / e.sum(axis=1, keepdims=True)
    ref = (p * masks[0][0][:, :5] * c) @ v[:5, 0]
    assert np.max(np.abs(o[:, 0] - ref)) < 1e-13
