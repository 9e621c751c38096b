"""Padded <-> unpadded storage on the GPU against oracle/unpad.py: bit-exact (integer and
copy work), through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import oracle, unpad
from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl
from gpu_util import oracle_inputs, to_f64

pytestmark = pytest.mark.gpu

RNG = np.random.default_rng(172)


def prefix_mask(lengths, s):
    m = np.zeros((len(lengths), s), dtype=np.int32)
    for i, n in enumerate(lengths):
        m[i, :n] = 1
    return m


def device_indices(m):
    nb, s = m.shape
    dm = torch.from_numpy(m).cuda()
    idx = torch.full((nb * s,), -7, dtype=torch.int32, device="cuda")
    inv = torch.full((nb * s,), -7, dtype=torch.int32, device="cuda")
    cu = torch.full((nb + 1,), -7, dtype=torch.int32, device="cuda")
    fmha.fmha_unpad_indices(dm, idx, inv, cu)
    torch.cuda.synchronize()
    return idx, inv, cu


def masks():
    yield "one", np.ones((1, 1), dtype=np.int32)
    yield "ragged_tail", prefix_mask([3, 17, 64, 65, 0, 130], 130)
    yield "holes", (RNG.integers(-2, 3, size=(37, 200)) * (RNG.random((37, 200)) < 0.5)).astype(np.int32)
    yield "empty_rows", np.zeros((5, 70), dtype=np.int32)
    yield "workload3", prefix_mask(wl.make_workload(3)["lengths"], 512)
    yield "many_rows", prefix_mask(RNG.integers(0, 513, size=2500), 512)   # more rows than scan threads
    yield "no_columns", np.zeros((4, 0), dtype=np.int32)
    yield "no_rows", np.zeros((0, 16), dtype=np.int32)


@pytest.mark.parametrize("name,m", list(masks()), ids=[n for n, _ in masks()])
def test_device_indices_bit_exact(name, m):
    idx, inv, cu = device_indices(m)
    ridx, rinv, rcu = unpad.unpad_indices(m)
    n = len(ridx)
    assert np.array_equal(cu.cpu().numpy(), rcu)
    assert np.array_equal(idx.cpu().numpy()[:n], ridx)
    assert (idx.cpu().numpy()[n:] == -7).all(), "entries beyond the count were written"
    assert np.array_equal(inv.cpu().numpy(), rinv)


@pytest.mark.parametrize("row_elems", [8, 64, 1024, 1032])
def test_gather_scatter_bit_exact(row_elems):
    lengths = [5, 0, 128, 77, 1]
    s = 128
    m = prefix_mask(lengths, s)
    m[3, 10] = 0                                   # a hole: nothing assumes prefixes
    ridx, rinv, rcu = unpad.unpad_indices(m)
    idx, inv, cu = device_indices(m)
    rows = m.size
    x = RNG.integers(0, 2 ** 16, size=(rows, row_elems)).astype(np.uint16)
    dx = torch.from_numpy(x.view(np.int16)).cuda()
    packed = torch.full((rows, row_elems), 0x5555, dtype=torch.int16, device="cuda")   # worst-case room
    fmha.fmha_gather_rows(dx, idx, cu[-1:], packed)
    torch.cuda.synchronize()
    n = len(ridx)
    want = unpad.gather_rows(x, ridx)
    got = packed.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[:n], want)
    assert (got[n:] == 0x5555).all(), "rows beyond the token count were written"
    back = torch.full((rows, row_elems), 0x3333, dtype=torch.int16, device="cuda")
    fmha.fmha_scatter_rows(packed, inv, cu[-1:], back)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy().view(np.uint16), unpad.scatter_rows(want, ridx, rows))


def test_out_of_range_indices_give_zero_rows():
    x = torch.arange(4 * 8, dtype=torch.int16, device="cuda").reshape(4, 8) + 1
    idx = torch.tensor([2, -1, 4, 0], dtype=torch.int32, device="cuda")
    n = torch.tensor([4], dtype=torch.int32, device="cuda")
    out = torch.full((4, 8), -1, dtype=torch.int16, device="cuda")
    fmha.fmha_gather_rows(x, idx, n, out)
    inv = torch.tensor([1, 9, -1, 0], dtype=torch.int32, device="cuda")
    back = torch.full((4, 8), -1, dtype=torch.int16, device="cuda")
    fmha.fmha_scatter_rows(x, inv, n, back)
    torch.cuda.synchronize()
    assert torch.equal(out[0], x[2]) and torch.equal(out[3], x[0]) and (out[1] == 0).all() and (out[2] == 0).all()
    assert torch.equal(back[0], x[1]) and torch.equal(back[3], x[0]) and (back[1] == 0).all() and (back[2] == 0).all()


def test_empty_row_copies_are_accepted():
    lib = fmha.lib()
    assert lib.fmha_gather_rows(None, 0, None, None, 0, 0, None, None) == fmha.FMHA_OK
    assert lib.fmha_scatter_rows(None, 0, None, None, 0, 0, None, None) == fmha.FMHA_OK


def test_row_copy_argument_errors():
    x = torch.zeros((4, 8), dtype=torch.int16, device="cuda")
    idx = torch.zeros(4, dtype=torch.int32, device="cuda")
    lib = fmha.lib()
    bad = lib.fmha_gather_rows(x.data_ptr(), 4, idx.data_ptr(), idx.data_ptr(), 4, 24, x.data_ptr(), None)
    assert bad == fmha.FMHA_ERR_INVALID_ARG and "multiple of 16" in fmha.last_error()
    bad = lib.fmha_scatter_rows(x.data_ptr() + 2, 4, idx.data_ptr(), idx.data_ptr(), 4, 16, x.data_ptr(), None)
    assert bad == fmha.FMHA_ERR_INVALID_ARG
    bad = lib.fmha_gather_rows(None, 4, idx.data_ptr(), idx.data_ptr(), 4, 16, x.data_ptr(), None)
    assert bad == fmha.FMHA_ERR_INVALID_ARG


def test_padded_input_through_gather_attention_scatter():
    """The paper's data flow (Section IV-A-1): padded input -> gather -> unpadded attention
    -> scatter -> padded output, everything on the device with no host synchronisation in
    between, against the oracle on the packed data."""
    lengths = [100, 512, 3, 257, 64]
    b = wl.make_batch(lengths, 4, "f16", seed=77)
    pb = wl.pad_batch(b, 512)
    h, rows = b["heads"], 5 * 512
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.float16)
    mask = torch.from_numpy(prefix_mask(lengths, 512)).cuda()
    idx = torch.empty(rows, dtype=torch.int32, device="cuda")
    inv = torch.empty(rows, dtype=torch.int32, device="cuda")
    cu = torch.empty(6, dtype=torch.int32, device="cuda")
    fmha.fmha_unpad_indices(mask, idx, inv, cu)
    t = b["total_tokens"]                       # known to the test, not needed by the kernels
    packed = {}
    for name in ("q", "k", "v"):
        packed[name] = torch.zeros((rows, h, 64), dtype=torch.float16, device="cuda")   # worst-case room
        fmha.fmha_gather_rows(dev(pb[name]), idx, cu[-1:], packed[name])
    q, k, v = (packed[n][:t] for n in ("q", "k", "v"))
    o = torch.empty_like(q)
    lse = torch.empty((h, t), dtype=torch.float32, device="cuda")
    ws = fmha.alloc_workspace(5, t, h, False)
    fmha.fmha_varlen_fwd(q, k, v, cu, 512, b["scale"], o, lse, ws)
    o_pad = torch.full((rows, h, 64), float("nan"), dtype=torch.float16, device="cuda")
    fmha.fmha_scatter_rows(o, inv, cu[-1:], o_pad)
    torch.cuda.synchronize()
    x = oracle_inputs(b)
    o_ref, _ = oracle.fwd(x["q"], x["k"], x["v"], b["cu_seqlens"], b["scale"])
    want = unpad.scatter_rows(o_ref, unpad.unpad_indices(prefix_mask(lengths, 512))[0], rows)
    got = to_f64(o_pad)
    assert not np.isnan(got).any()
    assert np.abs(got - want).max() <= 5e-3
    valid = prefix_mask(lengths, 512).ravel() != 0
    assert (got[~valid] == 0).all()
