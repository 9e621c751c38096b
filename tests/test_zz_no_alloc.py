"""fmha_varlen_fwd_static (the forward entry point that allocates nothing: its tile list lives
in a device array inside the library) against fmha_varlen_fwd, through the C ABI.  Both run
the same kernels, so O and LSE must agree bit for bit, which is within the forward's bar
(max-abs 5e-3 on O).  Two calls in a row on the same GPU, the second on a smaller batch: the
array still holds the first call's longer tile list when the second call starts."""
import numpy as np
import pytest
import torch

from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl
from tests.gpu_util import DeviceBatch

pytestmark = pytest.mark.gpu


def run_both(lengths, heads, dtype, seed):
    b = wl.make_batch(lengths, heads, dtype, seed=seed)
    d = DeviceBatch(b, need_bwd=False)
    d.fwd()
    o_ref, lse_ref = d.o.clone(), d.lse.clone()
    d.o.fill_(float("nan"))
    d.lse.fill_(float("nan"))
    fmha.fmha_varlen_fwd_static(d.q, d.k, d.v, d.cu, b["max_seqlen"], b["scale"], d.o, d.lse,
                                seqused=d.seqused)
    torch.cuda.synchronize()
    return d, o_ref, lse_ref


def same_bits(a, b):
    return torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_static_forward_matches_workspace_forward_twice():
    # first call: 40 sequences, several tiles each, ragged tails; second call: fewer and shorter
    big = [512, 300, 1, 129, 64, 200, 511, 33, 128, 257] * 4
    small = [70, 5, 130]
    for lengths, heads, dtype, seed in ((big, 4, "f16", 11), (small, 2, "f16", 12), (small, 3, "bf16", 13)):
        d, o_ref, lse_ref = run_both(lengths, heads, dtype, seed)
        assert not torch.isnan(d.o.float()).any()
        assert same_bits(d.o, o_ref), (len(lengths), heads, dtype)
        assert torch.equal(d.lse.view(torch.int32), lse_ref.view(torch.int32))
        err = (d.o.double() - o_ref.double()).abs().max().item()
        assert err <= 5e-3


def test_static_forward_reuses_its_own_list_and_rejects_oversize():
    lengths = [100, 260, 17]
    d, o_ref, lse_ref = run_both(lengths, 2, "f16", 21)
    b = d.b
    d.o.fill_(float("nan"))
    fmha.fmha_varlen_fwd_static(d.q, d.k, d.v, d.cu, b["max_seqlen"], b["scale"], d.o, d.lse,
                                reuse_schedule=True)
    torch.cuda.synchronize()
    assert same_bits(d.o, o_ref)
    # beyond the built-in array: rejected on the host, nothing launched
    limit = fmha.lib().fmha_varlen_static_scratch_bytes()
    assert limit == 1 << 20
    p = fmha.Params()
    p.batch, p.total_tokens, p.heads, p.head_dim, p.max_seqlen = 70000, 70000, 1, 64, 1
    p.dtype, p.scale = fmha.FMHA_F16, 0.125
    assert fmha.fmha_varlen_workspace_size(p.batch, p.total_tokens, p.heads, False) > limit
    rc = fmha.lib().fmha_varlen_fwd_static(p, d.q.data_ptr(), d.k.data_ptr(), d.v.data_ptr(), d.o.data_ptr(),
                                           d.lse.data_ptr(), None)
    assert rc == fmha.FMHA_ERR_WORKSPACE and "built-in scratch" in fmha.last_error()
