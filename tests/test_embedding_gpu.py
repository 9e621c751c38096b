"""Embedding backward on the GPU against oracle/embedding.py, through the C ABI.

The additions are atomic adds in the 16-bit type in an order that is not fixed, so several
results are correct.  What is unique is checked exactly (rows that receive zero or one
gradient row); the rest must be valid: within n half-ulps of the bound A = sum |terms| on
any partial sum (n = number of rows received; every addition rounds to nearest), and, as a
sharper aggregate check, the errors relative to sqrt(n) ulps must be O(1) on average."""
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
    bound = (cnt + 1)[:, None] * ulp_half(a, dtype) * 2 + 1e-30          # n half-ulps at A (ulp_half is at most 2x low at binade edges)
    assert (err <= bound).all(), f"max error / bound = {(err / bound).max():.3f}"
    many = cnt >= 4
    if many.any():
        typical = err[many] / (np.sqrt(cnt[many])[:, None] * 2 * ulp_half(np.maximum(np.abs(want[many]), 1e-3), dtype))
        assert typical.mean() < 2.0, f"mean error in sqrt(n) ulps: {typical.mean():.2f}"
    return got


SPLITS = ["default", "merged_no_die_split", "plain"]


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


@pytest.mark.parametrize("split", ["default", "merged_no_die_split"])
@pytest.mark.parametrize("dtype,vocab", [("f16", 30522), ("bf16", 997)])
def test_embedding_bwd_large_batch_uses_wide_windows(dtype, vocab, split):
    """From 2^17 rows on the workgroups look at 256 tokens at a time (four ids per lane)."""
    run_case(140001, 64, vocab, dtype, seed=17, split=split)


def test_embedding_bwd_one_hot_row_all_tokens_collide():
    """Every token has the same id: the worst case for the atomics."""
    ids = np.full(2000, 17, dtype=np.int32)
    run_case(2000, 256, 32, "f16", seed=2, split="default", ids=ids)


def test_embedding_bwd_argument_errors():
    dy = torch.zeros((4, 12), dtype=torch.float16, device="cuda")
    idx = torch.zeros(4, dtype=torch.int32, device="cuda")
    dw = torch.zeros((3, 12), dtype=torch.float16, device="cuda")
    with pytest.raises(fmha.FmhaError) as e:
        fmha.fmha_embedding_bwd(dy, idx, dw)
    assert e.value.code == fmha.FMHA_ERR_INVALID_ARG and "multiple of 8" in str(e.value)
