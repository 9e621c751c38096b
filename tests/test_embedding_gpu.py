"""Embedding backward on the GPU against oracle/embedding.py, through the C ABI.

In fmha_embedding_bwd the additions are atomic adds in the 16-bit type in an order that is not
fixed, so several results are correct.  What is unique is checked exactly (rows that receive zero or one
gradient row); the rest must be valid: within n half-ulps of the bound A = sum |terms| on
any partial sum (n = number of rows received; every addition rounds to nearest), and, as a
sharper aggregate check, the errors relative to sqrt(n) ulps must be O(1) on average.

The sorted variant (fmha_embedding_sort + fmha_embedding_bwd_sorted, split "sorted" below) sums
in fp32 in a fixed order and rounds once: its results are unique.  They are checked against
the oracle with the bound of an fp32 sum plus one rounding, against a numpy restatement of its
summation order bit for bit, and for identical reruns."""
import numpy as np
import pytest
import torch

from oracle import embedding as emb
from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl
from gpu_util import TORCH_DT, to_dev, to_f64, ulp_half

pytestmark = pytest.mark.gpu


def run_case(t, n, vocab, dtype, seed, *, split, padding_idx=-1, init=False, cap=None, ids=None):
    rng = np.random.default_rng(seed)
    cap = t if cap is None else cap
    dy_bits = wl.to_bits(rng.standard_normal((cap, n)).astype(np.float32), dtype)
    ids = wl.zipf_token_ids(cap, vocab, seed + 1) if ids is None else ids
    dy = to_dev(dy_bits, dtype)
    idx = torch.from_numpy(ids).cuda()
    if init:
        w0 = wl.to_bits(rng.standard_normal((vocab, n)).astype(np.float32), dtype)
        dw = to_dev(w0, dtype)
    else:
        w0 = None
        dw = torch.full((vocab, n), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    n_rows = torch.tensor([t], dtype=torch.int32, device="cuda") if cap != t else None
    if split == "sorted":
        ws = torch.empty(fmha.fmha_embedding_sort_workspace_size(cap, n), dtype=torch.uint8, device="cuda")
        fmha.fmha_embedding_sort(idx, n, vocab, ws, padding_idx=padding_idx, n_rows=n_rows)
        fmha.fmha_embedding_bwd_sorted(dy, ws, dw, zero_first=not init)
    else:
        fmha.fmha_embedding_bwd(dy, idx, dw, padding_idx=padding_idx, n_rows=n_rows, zero_first=not init,
                                plain_split=split == "plain", no_die_split=split == "merged_no_die_split")
    torch.cuda.synchronize()
    got = to_f64(dw)
    x = wl.bits_to_f64(dy_bits[:t], dtype)
    init64 = None if w0 is None else wl.bits_to_f64(w0, dtype)
    want, cnt = emb.embedding_bwd(x, ids[:t], vocab, padding_idx, init64)
    a = emb.abs_sums(x, ids[:t], vocab, padding_idx) + (0 if init64 is None else np.abs(init64))
    assert not np.isnan(got).any()
    zero = cnt == 0
    assert np.array_equal(got[zero], want[zero]), "rows that receive nothing must be untouched / zero"
    if not init:
        one = cnt == 1
        assert np.array_equal(got[one], want[one]), "a single contribution must arrive exactly"
    err = np.abs(got - want)
    if split == "sorted":
        # an fp32 sum of n + 1 terms (each addition within 2^-24 of the partial sum, itself at most
        # A) and one rounding to the 16-bit type at the result
        bound = (cnt + 1)[:, None] * a * 2.0 ** -24 + ulp_half(np.abs(want) + (cnt + 1)[:, None] * a * 2.0 ** -24, dtype) * 2 + 1e-30
    else:
        bound = (cnt + 1)[:, None] * ulp_half(a, dtype) * 2 + 1e-30      # n half-ulps at A (ulp_half is at most 2x low at binade edges)
    assert (err <= bound).all(), f"max error / bound = {(err / bound).max():.3f}"
    many = cnt >= 4
    if many.any():
        typical = err[many] / (np.sqrt(cnt[many])[:, None] * 2 * ulp_half(np.maximum(np.abs(want[many]), 1e-3), dtype))
        assert typical.mean() < 2.0, f"mean error in sqrt(n) ulps: {typical.mean():.2f}"
    return got


SPLITS = ["default", "merged_no_die_split", "plain", "sorted"]


@pytest.mark.parametrize("split", SPLITS)
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("t,n,vocab", [(1, 8, 3), (70, 64, 50), (1000, 768, 997), (5000, 1024, 30522), (300, 1032, 64)])
def test_embedding_bwd(t, n, vocab, dtype, split):
    run_case(t, n, vocab, dtype, seed=t + n, split=split)


@pytest.mark.parametrize("split", SPLITS)
def test_embedding_bwd_accumulates_skips_and_respects_the_row_count(split):
    ids = wl.zipf_token_ids(400, 40, 5)
    ids[::7] = -3          # out of range: skipped
    ids[3::11] = 40        # out of range: skipped
    run_case(250, 128, 40, "f16", seed=8, split=split, padding_idx=int(ids[1]), init=True, cap=400, ids=ids)


@pytest.mark.parametrize("split", ["default", "merged_no_die_split", "sorted"])
@pytest.mark.parametrize("dtype,vocab", [("f16", 30522), ("bf16", 997)])
def test_embedding_bwd_large_batch_uses_wide_windows(dtype, vocab, split):
    """From 2^17 rows on the workgroups look at 256 tokens at a time (four ids per lane; the
    sorted variant takes 256 sorted entries per workgroup instead of 32)."""
    run_case(140001, 64, vocab, dtype, seed=17, split=split)


def test_embedding_bwd_one_hot_row_all_tokens_collide():
    """Every token has the same id: the worst case for the atomics."""
    ids = np.full(2000, 17, dtype=np.int32)
    run_case(2000, 256, 32, "f16", seed=2, split="default", ids=ids)


def test_embedding_bwd_one_hot_row_sorted():
    """Every token has the same id: one run across all chunks, combined in chunk order."""
    ids = np.full(2000, 17, dtype=np.int32)
    run_case(2000, 256, 32, "bf16", seed=3, split="sorted", ids=ids)


def sorted_order_reference(dy_bits, ids, vocab, dtype, chunk, init_bits=None):
    """The sorted variant's arithmetic restated with numpy float32: stable sort by index, chunks
    of `chunk` sorted entries, inside a chunk every run summed row by row, the partial sums of a
    run that spans chunks added in chunk order, the old weight row added last, one rounding."""
    x = wl.bits_to_f64(dy_bits, dtype).astype(np.float32)
    keep = (ids >= 0) & (ids < vocab)
    order = np.argsort(np.where(keep, ids, vocab), kind="stable")
    out = np.zeros((vocab, x.shape[1]), np.float32) if init_bits is None else wl.bits_to_f64(init_bits, dtype).astype(np.float32)
    sums = {}
    for c0 in range(0, len(order), chunk):
        part = {}
        for pos in order[c0:c0 + chunk]:
            if keep[pos]:
                k = int(ids[pos])
                part[k] = part.get(k, np.zeros(x.shape[1], np.float32)) + x[pos]
        for k, v in part.items():
            sums[k] = v if k not in sums else sums[k] + v
    for k, v in sums.items():
        out[k] = out[k] + v if init_bits is not None else v
    return wl.to_bits(out, dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("t,n,vocab,init", [(900, 72, 11, False), (3000, 768, 301, True)])
def test_sorted_variant_bit_for_bit_and_repeatable(t, n, vocab, init, dtype):
    rng = np.random.default_rng(t)
    dy_bits = wl.to_bits(rng.standard_normal((t, n)).astype(np.float32), dtype)
    ids = wl.zipf_token_ids(t, vocab, 9)
    ids[5::13] = -1
    w0 = wl.to_bits(rng.standard_normal((vocab, n)).astype(np.float32), dtype) if init else None
    dy, idx = to_dev(dy_bits, dtype), torch.from_numpy(ids).cuda()
    ws = torch.empty(fmha.fmha_embedding_sort_workspace_size(t, n), dtype=torch.uint8, device="cuda")
    fmha.fmha_embedding_sort(idx, n, vocab, ws)
    results = []
    for _ in range(2):   # the sorted positions serve any number of backward calls
        dw = to_dev(w0, dtype) if init else torch.full((vocab, n), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
        fmha.fmha_embedding_bwd_sorted(dy, ws, dw, zero_first=not init)
        torch.cuda.synchronize()
        results.append(dw.view(torch.int16).cpu().numpy().view(np.uint16))
    assert np.array_equal(results[0], results[1])
    want = sorted_order_reference(dy_bits, ids, vocab, dtype, 32, w0)   # batches under 2^17 rows: chunks of 32
    assert np.array_equal(results[0], want)


def test_embedding_bwd_argument_errors():
    dy = torch.zeros((4, 12), dtype=torch.float16, device="cuda")
    idx = torch.zeros(4, dtype=torch.int32, device="cuda")
    dw = torch.zeros((3, 12), dtype=torch.float16, device="cuda")
    with pytest.raises(fmha.FmhaError) as e:
        fmha.fmha_embedding_bwd(dy, idx, dw)
    assert e.value.code == fmha.FMHA_ERR_INVALID_ARG and "multiple of 8" in str(e.value)
