"""Attention-probability dropout on the GPU against the CPU oracle.

The keep mask is a function of (seed, sequence start, head, query, key) that the
library and oracle/dropout_mask.py implement independently: first the mask
itself is compared bit for bit (in both of the kernels' tile orientations),
then outputs and gradients to the same tolerances as without dropout.
"""
import numpy as np
import pytest
import torch

from oracle import dropout_mask as dm
from oracle import oracle
from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl
from gpu_util import DeviceBatch, oracle_inputs, to_f64, ulp_half

pytestmark = pytest.mark.gpu

O_TOL = 5e-3
G_TOL = 1e-2
G_FLOOR = 0.1


def gpu_mask(lengths, heads, p, seed, orientation):
    cu_np = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    cu = torch.from_numpy(cu_np).cuda()
    t, lmax = int(cu_np[-1]), max(max(lengths), 1)
    mask = torch.full((heads, t, lmax), 7, dtype=torch.uint8, device="cuda")
    ws = fmha.alloc_workspace(len(lengths), t, heads, False)
    fmha.fmha_dropout_keep_mask(heads, cu, lmax, (p, seed), mask, ws, orientation=orientation,
                                cu_seqlens_host=torch.from_numpy(cu_np))
    torch.cuda.synchronize()
    return cu_np, mask.cpu().numpy()


@pytest.mark.parametrize("orientation", [0, 1])
@pytest.mark.parametrize("lengths,heads,p,seed", [
    ([3, 17, 64, 128], 2, 0.1, 1),
    ([200, 1, 77, 0, 333], 3, 0.5, 0xDEADBEEFCAFEF00D),
    ([640], 1, 0.9, 2 ** 63 + 12345),
])
def test_keep_mask_bit_exact(lengths, heads, p, seed, orientation):
    cu, got = gpu_mask(lengths, heads, p, seed, orientation)
    want = dm.keep_masks(cu, heads, p, seed)
    for i, n in enumerate(lengths):
        if n == 0:
            continue
        blk = got[:, cu[i]:cu[i + 1], :]
        assert np.array_equal(blk[:, :, :n], want[i]), f"sequence {i} (L={n})"
        assert (blk[:, :, n:] == 7).all(), "bytes beyond the sequence's keys were written"


def check(b, db, p, seed):
    x = oracle_inputs(b)
    cu = b["cu_seqlens"]
    masks = dm.keep_masks(cu, b["heads"], p, seed)
    c = dm.keep_scale(p)
    su = b.get("seqused")
    o_ref, lse_ref = oracle.fwd_dropout(x["q"], x["k"], x["v"], cu, b["scale"], masks, c, su)
    o, lse = to_f64(db.o), to_f64(db.lse)
    assert not np.isnan(o).any() and not np.isnan(lse).any()
    extra = ulp_half(o_ref, b["dtype"]) if b["dtype"] == "bf16" else 0.0
    err = np.abs(o - o_ref)
    assert (err <= O_TOL + extra).all(), f"max |O - O_ref| = {err.max():.3e}"
    fin = np.isfinite(lse_ref)
    assert np.abs(lse[fin] - lse_ref[fin]).max() <= 1e-3 * max(1.0, np.abs(lse_ref[fin]).max())
    if db.do is None:
        return
    ref = oracle.bwd_dropout(x["q"], x["k"], x["v"], x["do"], cu, b["scale"], masks, c, su)
    # Rows of single-token sequences are left out of the dQ / dK comparison: their exact
    # gradient is zero by cancellation of two O(10) terms, one of which the kernels form from
    # the stored 16-bit O (= V / (1-p), no longer exact as it is without dropout), so what
    # remains is that rounding - up to 1e-2 absolute in bfloat16, which would be measured
    # against the small gradients of long sequences.  test_single_token_sequences_under_dropout
    # bounds those rows by what the rounding of O allows.
    # Every sequence is measured on its own scale (max-abs error over its rows / max |reference|
    # over the same rows, floored at G_FLOOR).
    for name, got, want in zip(("dq", "dk", "dv"), (db.dq, db.dk, db.dv), ref):
        g = to_f64(got)
        assert not np.isnan(g).any(), f"{name}: rows left unwritten"
        for i in range(len(cu) - 1):
            a, e = int(cu[i]), int(cu[i + 1])
            if e == a or (e - a == 1 and name != "dv"):
                continue
            rel = np.abs(g[a:e] - want[a:e]).max() / max(np.abs(want[a:e]).max(), G_FLOOR)
            assert rel <= G_TOL, f"{name}, sequence {i}: max-abs error / max|ref| = {rel:.3e}"


def run(b, p, seed, need_bwd=True):
    db = DeviceBatch(b, need_bwd)
    db.fwd(dropout=(p, seed))
    if need_bwd:
        db.bwd(reuse_schedule=True, dropout=(p, seed))
    torch.cuda.synchronize()
    check(b, db, p, seed)
    return db


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("lengths,p", [
    ([1], 0.1), ([2, 1, 3], 0.5), ([31, 32, 33], 0.1), ([63, 64, 65], 0.25), ([127, 128, 129], 0.1),
    ([200, 5, 77, 300], 0.1), ([512, 1, 511, 257], 0.1), ([0, 40, 0, 0, 7, 0], 0.3), ([640, 130], 0.1),
])
def test_dropout_fwd_bwd_ragged(lengths, p, dtype):
    b = wl.make_batch(lengths, 3, dtype, seed=sum(lengths) + len(lengths) + 1000)
    run(b, p, seed=977 * sum(lengths) + 5)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_single_token_sequences_under_dropout(dtype):
    """L = 1: P = 1, so O = V / (1-p) if the one element is kept and 0 if not, dV likewise
    from dO, and dQ = dK = 0 in exact arithmetic.  The kernels form D from the stored
    (16-bit) O, so dS = dP - D is what that rounding leaves:
        |dS| <= sum_c |dO_c| * (half an ulp of O_c)  +  fp32 effects,
    and |dQ| <= |scale| max|K| |dS|, the same with Q for dK.  The fp32 effects (two 64-term
    dot products accumulated in fp32, relative error <= 64 * 2^-24 each, and the exponent's
    argument, |P - 1| <= 3 * 2^-24 |S log2 e|) are bounded by 2.2e-5 * sum_c |dO_c O_c|, which
    is at most 2.2e-5 * 2^12 = 9 % of the first term (|O| / half-ulp(O) <= 2^12 for f16, 2^9
    for bf16); the 16-bit roundings of dS and of the stored dQ add under 1 %.  Hence the
    factor 1.15 below and no additive term: a dropped element has O = 0, D = dP = 0 and an
    exactly zero gradient."""
    n, h, p, seed = 40, 2, 0.5, 77
    b = wl.make_batch([1] * n, h, dtype, seed=11)
    db = DeviceBatch(b, True)
    db.fwd(dropout=(p, seed))
    db.bwd(reuse_schedule=True, dropout=(p, seed))
    torch.cuda.synchronize()
    x = oracle_inputs(b)
    c = dm.keep_scale(p)
    keep = np.stack([dm.keep_masks(b["cu_seqlens"], h, p, seed)[i][:, 0, 0] for i in range(n)])  # [n, h]
    assert 0 < keep.sum() < keep.size
    o, dq, dk, dv = (to_f64(t) for t in (db.o, db.dq, db.dk, db.dv))
    o_want = x["v"] * (keep * c)[:, :, None]
    assert (np.abs(o - o_want) <= ulp_half(o_want, dtype) + 1e-12).all()
    dv_want = x["do"] * (keep * c)[:, :, None]
    assert (np.abs(dv - dv_want) <= ulp_half(dv_want, dtype) * 1.01 + 1e-12).all()
    half_ulp_o = ulp_half(o_want, dtype).max(axis=2)                       # [n, h]
    slack = abs(b["scale"]) * np.abs(x["do"]).sum(axis=2) * half_ulp_o * 1.15
    assert (np.abs(dq) <= (np.abs(x["k"]).max(axis=2) * slack)[:, :, None]).all()
    assert (np.abs(dk) <= (np.abs(x["q"]).max(axis=2) * slack)[:, :, None]).all()


def test_dropout_config1():
    b = wl.make_workload(1)
    run(b, 0.1, seed=220808124, need_bwd=False)


def test_dropout_with_seqused_and_strides():
    """Padded layout with a key mask, interleaved QKV storage, and dropout together."""
    lengths = [96, 130, 17]
    b = wl.make_batch(lengths, 2, "f16", seed=4242)
    b["seqused"] = np.array([50, 130, 0], dtype=np.int32)
    db = DeviceBatch(b, True)
    t, h = b["total_tokens"], b["heads"]
    qkv = torch.empty((t, 3, h, 64), dtype=torch.float16, device="cuda")
    qkv[:, 0], qkv[:, 1], qkv[:, 2] = db.q, db.k, db.v
    db.q, db.k, db.v = qkv[:, 0], qkv[:, 1], qkv[:, 2]
    db.fwd(dropout=(0.2, 31337))
    db.bwd(reuse_schedule=True, dropout=(0.2, 31337))
    torch.cuda.synchronize()
    check(b, db, 0.2, 31337)


def test_p_zero_is_the_plain_path_bitwise():
    b = wl.make_batch([130, 64, 7], 2, "f16", seed=99)
    a, c = DeviceBatch(b, True), DeviceBatch(b, True)
    a.fwd(); a.bwd(reuse_schedule=True)
    c.fwd(dropout=(0.0, 5)); c.bwd(reuse_schedule=True, dropout=(0.0, 5))
    torch.cuda.synchronize()
    for n in ("o", "lse", "dq", "dk", "dv"):
        assert torch.equal(getattr(a, n), getattr(c, n)), n


def test_dropout_is_deterministic_and_seed_dependent():
    b = wl.make_batch([257, 64], 2, "f16", seed=5)
    r1 = run(b, 0.1, seed=1)
    r2 = run(b, 0.1, seed=1)
    r3 = run(b, 0.1, seed=2)
    for n in ("o", "dq", "dk", "dv"):
        assert torch.equal(getattr(r1, n), getattr(r2, n)), n
    assert not torch.equal(r1.o, r3.o)
    assert torch.equal(r1.lse, r3.lse)   # the softmax statistics do not see the mask


def test_dropout_bad_arguments():
    b = wl.make_batch([16], 1, "f16", seed=1)
    db = DeviceBatch(b, False)
    for bad in (1.0, -0.1, float("nan")):
        with pytest.raises(fmha.FmhaError) as e:
            db.fwd(dropout=(bad, 1))
        assert e.value.code == fmha.FMHA_ERR_INVALID_ARG


def test_dropout_bert_large_batch_sampled():
    """The benchmark's batch (workload 3) with p = 0.1, checked against the oracle on a
    sample of sequences run as their own small batches: the mask depends on a sequence's
    start row, so the sample is compared through the mask bytes the oracle generates for
    the same start rows."""
    b = wl.make_workload(3)
    p, seed = 0.1, 2208
    db = DeviceBatch(b, True)
    db.fwd(dropout=(p, seed))
    db.bwd(reuse_schedule=True, dropout=(p, seed))
    torch.cuda.synchronize()
    cu, h = b["cu_seqlens"], b["heads"]
    lens = np.diff(cu)
    pick = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 0, len(lens) - 1, len(lens) // 2})
    x = oracle_inputs(b)
    c = dm.keep_scale(p)
    t = dm.threshold(p)
    for i in pick:
        sl = slice(int(cu[i]), int(cu[i + 1]))
        n = int(lens[i])
        m = [(dm.random_bytes(int(cu[i]), h, n, n, seed) >= t).astype(np.uint8)]
        cu1 = np.array([0, n], dtype=np.int32)
        o_ref, _ = oracle.fwd_dropout(x["q"][sl], x["k"][sl], x["v"][sl], cu1, b["scale"], m, c)
        g_ref = oracle.bwd_dropout(x["q"][sl], x["k"][sl], x["v"][sl], x["do"][sl], cu1, b["scale"], m, c)
        assert np.abs(to_f64(db.o[sl]) - o_ref).max() <= O_TOL, f"sequence {i}"
        for name, got, want in zip(("dq", "dk", "dv"), (db.dq, db.dk, db.dv), g_ref):
            rel = np.abs(to_f64(got[sl]) - want).max() / max(np.abs(want).max(), G_FLOOR)
            assert rel <= G_TOL, f"sequence {i} {name}: {rel:.3e}"


def test_dropout_large_batch_bf16_sampled():
    """Workload 5 (2048 sequences, 12 heads, bf16) with p = 0.1 at the benchmark's launch
    configuration; a sample of sequences with more than one token is checked against the
    oracle, each with the mask the oracle generates for its start row."""
    b = wl.make_workload(5)
    p, seed = 0.1, 55
    db = DeviceBatch(b, True)
    db.fwd(dropout=(p, seed))
    db.bwd(reuse_schedule=True, dropout=(p, seed))
    torch.cuda.synchronize()
    for t_ in (db.o, db.dq, db.dk, db.dv, db.lse):
        assert not torch.isnan(t_).any(), "rows left unwritten"
    cu, h, L = b["cu_seqlens"], b["heads"], b["lengths"]
    rng = np.random.default_rng(6)
    cand = [i for i in rng.choice(len(L), 40, replace=False).tolist() if L[i] > 1][:10]
    pick = sorted(set(cand) | {int(L.argmax()), len(L) - 1 if L[-1] > 1 else int(L.argmax())})
    x = oracle_inputs(b)
    c, thr = dm.keep_scale(p), dm.threshold(p)
    for i in pick:
        sl = slice(int(cu[i]), int(cu[i + 1]))
        n = int(L[i])
        m = [(dm.random_bytes(int(cu[i]), h, n, n, seed) >= thr).astype(np.uint8)]
        cu1 = np.array([0, n], dtype=np.int32)
        o_ref, _ = oracle.fwd_dropout(x["q"][sl], x["k"][sl], x["v"][sl], cu1, b["scale"], m, c)
        g_ref = oracle.bwd_dropout(x["q"][sl], x["k"][sl], x["v"][sl], x["do"][sl], cu1, b["scale"], m, c)
        err = np.abs(to_f64(db.o[sl]) - o_ref)
        assert (err <= O_TOL + ulp_half(o_ref, "bf16")).all(), f"sequence {i}: {err.max():.3e}"
        for name, got, want in zip(("dq", "dk", "dv"), (db.dq, db.dk, db.dv), g_ref):
            rel = np.abs(to_f64(got[sl]) - want).max() / max(np.abs(want).max(), G_FLOOR)
            assert rel <= G_TOL, f"sequence {i} {name}: {rel:.3e}"
