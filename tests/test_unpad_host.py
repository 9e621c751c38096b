"""The library's host routine for nonzero_indices / batch_offset against the oracle
(no GPU involved: plain host arrays through the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import unpad
from paper_2208_08124_amd import fmha

RNG = np.random.default_rng(171)


@pytest.mark.parametrize("shape,density", [((1, 1), 1.0), ((4, 7), 0.5), ((9, 64), 0.9), ((33, 130), 0.3), ((5, 0), 0.5), ((0, 8), 0.5)])
def test_host_indices_match_the_oracle(shape, density):
    m = (RNG.integers(1, 4, size=shape) * (RNG.random(shape) < density)).astype(np.int32)
    idx, inv, cu, mx = fmha.fmha_unpad_indices_host(torch.from_numpy(m))
    ridx, rinv, rcu = unpad.unpad_indices(m)
    assert np.array_equal(idx.numpy(), ridx)
    assert np.array_equal(inv.numpy(), rinv)
    assert np.array_equal(cu.numpy(), rcu)
    assert mx == (int(np.diff(rcu).max()) if shape[0] else 0)


def test_host_indices_reject_bad_sizes():
    lib = fmha.lib()
    cu = torch.zeros(4, dtype=torch.int32)
    assert lib.fmha_unpad_indices_host(None, -1, 4, None, None, cu.data_ptr(), None) == fmha.FMHA_ERR_INVALID_ARG
    assert lib.fmha_unpad_indices_host(None, 2, 4, None, None, cu.data_ptr(), None) == fmha.FMHA_ERR_INVALID_ARG
    assert lib.fmha_unpad_indices_host(None, 1 << 20, 1 << 20, None, None, cu.data_ptr(), None) == fmha.FMHA_ERR_INVALID_ARG
    assert "2^31" in fmha.last_error()
