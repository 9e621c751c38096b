"""ctypes binding of libfmha_varlen.so (see include/fmha_varlen.h).

Argument marshalling only: every step of the path runs in the HIP library.
torch is used for device memory and the current stream.  There is no CPU
fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfmha_varlen.so")

FMHA_OK, FMHA_ERR_INVALID_ARG, FMHA_ERR_UNSUPPORTED, FMHA_ERR_WORKSPACE, FMHA_ERR_HIP = range(5)
FMHA_F16, FMHA_BF16 = 0, 1
FMHA_FLAG_REUSE_SCHEDULE = 1
FMHA_FLAG_BWD_ONLY_DQ = 2
FMHA_FLAG_BWD_ONLY_DKV = 4
FMHA_EMB_ZERO_FIRST = 1
FMHA_EMB_PLAIN_SPLIT = 2
FMHA_EMB_NO_DIE_SPLIT = 4

EXPORTS = ("fmha_varlen_workspace_size", "fmha_varlen_fwd", "fmha_varlen_bwd",
           "fmha_varlen_fwd_static", "fmha_varlen_static_scratch_bytes",
           "fmha_varlen_fwd_dropout", "fmha_varlen_bwd_dropout", "fmha_dropout_keep_mask",
           "fmha_unpad_indices_host", "fmha_unpad_indices", "fmha_gather_rows", "fmha_scatter_rows",
           "fmha_dropout_add_ln_fwd", "fmha_dropout_add_ln_bwd", "fmha_dropout_add_ln_bwd_workspace_size",
           "fmha_embedding_bwd", "fmha_embedding_sort_workspace_size", "fmha_embedding_sort",
           "fmha_embedding_bwd_sorted",
           "fmha_varlen_schedule_info", "fmha_last_error")


class Params(ctypes.Structure):
    """Mirror of fmha_varlen_params_t."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("total_tokens", ctypes.c_int32), ("heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("max_seqlen", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("flags", ctypes.c_uint32), ("scale", ctypes.c_float),
        ("q_stride", ctypes.c_int64), ("k_stride", ctypes.c_int64),
        ("v_stride", ctypes.c_int64), ("o_stride", ctypes.c_int64),
        ("do_stride", ctypes.c_int64), ("dq_stride", ctypes.c_int64),
        ("dk_stride", ctypes.c_int64), ("dv_stride", ctypes.c_int64),
        ("cu_seqlens", ctypes.c_void_p), ("cu_seqlens_host", ctypes.c_void_p),
        ("seqused", ctypes.c_void_p), ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
    ]


class Dropout(ctypes.Structure):
    """Mirror of fmha_dropout_t."""
    _fields_ = [("p", ctypes.c_float), ("seed", ctypes.c_uint64)]


class LnParams(ctypes.Structure):
    """Mirror of fmha_ln_params_t."""
    _fields_ = [("rows", ctypes.c_int32), ("hidden", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("eps", ctypes.c_float), ("n_rows", ctypes.c_void_p), ("dropout", Dropout)]


class FmhaError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"fmha_varlen error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2208_08124_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.fmha_varlen_workspace_size.argtypes = [ctypes.c_int32] * 4
        L.fmha_varlen_workspace_size.restype = ctypes.c_size_t
        L.fmha_varlen_fwd.argtypes = [ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp]
        L.fmha_varlen_fwd.restype = ctypes.c_int
        L.fmha_varlen_fwd_static.argtypes = [ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp]
        L.fmha_varlen_fwd_static.restype = ctypes.c_int
        L.fmha_varlen_static_scratch_bytes.argtypes = []
        L.fmha_varlen_static_scratch_bytes.restype = ctypes.c_size_t
        L.fmha_varlen_bwd.argtypes = [ctypes.POINTER(Params)] + [vp] * 10
        L.fmha_varlen_bwd.restype = ctypes.c_int
        dp = ctypes.POINTER(Dropout)
        L.fmha_varlen_fwd_dropout.argtypes = [ctypes.POINTER(Params), dp, vp, vp, vp, vp, vp, vp]
        L.fmha_varlen_fwd_dropout.restype = ctypes.c_int
        L.fmha_varlen_bwd_dropout.argtypes = [ctypes.POINTER(Params), dp] + [vp] * 10
        L.fmha_varlen_bwd_dropout.restype = ctypes.c_int
        L.fmha_dropout_keep_mask.argtypes = [ctypes.POINTER(Params), dp, ctypes.c_int32, ctypes.c_int32, vp, vp]
        L.fmha_dropout_keep_mask.restype = ctypes.c_int
        i32 = ctypes.c_int32
        L.fmha_unpad_indices_host.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.fmha_unpad_indices_host.restype = ctypes.c_int
        L.fmha_unpad_indices.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.fmha_unpad_indices.restype = ctypes.c_int
        L.fmha_gather_rows.argtypes = [vp, i32, vp, vp, i32, ctypes.c_int64, vp, vp]
        L.fmha_gather_rows.restype = ctypes.c_int
        L.fmha_scatter_rows.argtypes = [vp, i32, vp, vp, i32, ctypes.c_int64, vp, vp]
        L.fmha_scatter_rows.restype = ctypes.c_int
        lp = ctypes.POINTER(LnParams)
        L.fmha_dropout_add_ln_fwd.argtypes = [lp] + [vp] * 9
        L.fmha_dropout_add_ln_fwd.restype = ctypes.c_int
        L.fmha_dropout_add_ln_bwd.argtypes = [lp] + [vp] * 10 + [ctypes.c_size_t, vp]
        L.fmha_dropout_add_ln_bwd.restype = ctypes.c_int
        L.fmha_dropout_add_ln_bwd_workspace_size.argtypes = [i32, i32]
        L.fmha_dropout_add_ln_bwd_workspace_size.restype = ctypes.c_size_t
        L.fmha_embedding_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, ctypes.c_uint32, vp, vp]
        L.fmha_embedding_bwd.restype = ctypes.c_int
        L.fmha_embedding_sort_workspace_size.argtypes = [i32, i32]
        L.fmha_embedding_sort_workspace_size.restype = ctypes.c_size_t
        L.fmha_embedding_sort.argtypes = [vp, vp, i32, i32, i32, i32, vp, ctypes.c_size_t, vp]
        L.fmha_embedding_sort.restype = ctypes.c_int
        L.fmha_embedding_bwd_sorted.argtypes = [vp, vp, ctypes.c_size_t, i32, i32, i32, i32, ctypes.c_uint32, vp, vp]
        L.fmha_embedding_bwd_sorted.restype = ctypes.c_int
        L.fmha_varlen_schedule_info.argtypes = [ctypes.c_int32] * 3 + [ctypes.POINTER(ctypes.c_size_t)] * 2
        L.fmha_varlen_schedule_info.restype = ctypes.c_int32
        L.fmha_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def last_error() -> str:
    return lib().fmha_last_error().decode()


def _check(rc):
    if rc != FMHA_OK:
        raise FmhaError(rc, last_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return FMHA_F16
    if t.dtype == torch.bfloat16:
        return FMHA_BF16
    raise FmhaError(FMHA_ERR_UNSUPPORTED, f"dtype {t.dtype}")


def _tok_stride(t: torch.Tensor) -> int:
    assert t.dim() == 3 and t.stride(2) == 1 and t.stride(1) == t.shape[2], \
        "tensors are [T, H, 64] with heads contiguous inside a token"
    return t.stride(0) if t.shape[0] > 1 else t.shape[1] * t.shape[2]


def fmha_varlen_workspace_size(batch: int, total_tokens: int, heads: int, need_bwd: bool) -> int:
    return int(lib().fmha_varlen_workspace_size(batch, total_tokens, heads, int(need_bwd)))


def fmha_varlen_schedule_info(batch: int, total_tokens: int, max_seqlen: int = 0):
    """(capacity in tiles, byte offset of the count, byte offset of the list)."""
    c, l = ctypes.c_size_t(), ctypes.c_size_t()
    cap = lib().fmha_varlen_schedule_info(batch, total_tokens, max_seqlen, ctypes.byref(c), ctypes.byref(l))
    return int(cap), int(c.value), int(l.value)


def alloc_workspace(batch: int, total_tokens: int, heads: int, need_bwd: bool, device="cuda"):
    n = max(fmha_varlen_workspace_size(batch, total_tokens, heads, need_bwd), 256)
    return torch.empty(n, dtype=torch.uint8, device=device)


def _params(q, cu_seqlens, max_seqlen, scale, workspace, seqused, cu_seqlens_host, reuse_schedule,
            extra_flags=0):
    p = Params()
    p.batch = cu_seqlens.numel() - 1
    p.total_tokens, p.heads, p.head_dim = q.shape
    p.max_seqlen = int(max_seqlen)
    p.dtype = _dtype_code(q)
    p.flags = (FMHA_FLAG_REUSE_SCHEDULE if reuse_schedule else 0) | extra_flags
    p.scale = float(scale)
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.is_cuda and cu_seqlens.is_contiguous()
    p.cu_seqlens = cu_seqlens.data_ptr()
    keep = []
    if cu_seqlens_host is not None:
        h = cu_seqlens_host.to(dtype=torch.int32, device="cpu").contiguous()
        keep.append(h)
        p.cu_seqlens_host = h.data_ptr()
    if seqused is not None:
        assert seqused.dtype == torch.int32 and seqused.is_cuda and seqused.is_contiguous()
        p.seqused = seqused.data_ptr()
    if workspace is not None:
        p.workspace = workspace.data_ptr()
        p.workspace_bytes = workspace.numel() * workspace.element_size()
    return p, keep


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dropout(dropout):
    """(p, seed) -> fmha_dropout_t"""
    p, seed = dropout
    return Dropout(float(p), int(seed) & 0xFFFFFFFFFFFFFFFF)


def fmha_varlen_fwd(q, k, v, cu_seqlens, max_seqlen, scale, o, lse, workspace, *,
                    seqused=None, cu_seqlens_host=None, reuse_schedule=False, dropout=None):
    """Enqueue the forward pass on torch's current stream; fills `o` and `lse` ([H, T] fp32).
    `dropout` = (p, seed) selects fmha_varlen_fwd_dropout."""
    p, keep = _params(q, cu_seqlens, max_seqlen, scale, workspace, seqused, cu_seqlens_host, reuse_schedule)
    p.q_stride, p.k_stride, p.v_stride, p.o_stride = map(_tok_stride, (q, k, v, o))
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.numel() == q.shape[0] * q.shape[1]
    ptrs = (q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), _stream())
    if dropout is None:
        _check(lib().fmha_varlen_fwd(ctypes.byref(p), *ptrs))
    else:
        d = _dropout(dropout)
        _check(lib().fmha_varlen_fwd_dropout(ctypes.byref(p), ctypes.byref(d), *ptrs))
    del keep


def fmha_varlen_fwd_static(q, k, v, cu_seqlens, max_seqlen, scale, o, lse, *,
                           seqused=None, cu_seqlens_host=None, reuse_schedule=False):
    """fmha_varlen_fwd without a workspace: the tile list lives in the library's own device array."""
    p, keep = _params(q, cu_seqlens, max_seqlen, scale, None, seqused, cu_seqlens_host, reuse_schedule)
    p.q_stride, p.k_stride, p.v_stride, p.o_stride = map(_tok_stride, (q, k, v, o))
    assert lse.dtype == torch.float32 and lse.is_contiguous() and lse.numel() == q.shape[0] * q.shape[1]
    _check(lib().fmha_varlen_fwd_static(ctypes.byref(p), q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                        lse.data_ptr(), _stream()))
    del keep


def fmha_varlen_bwd(q, k, v, o, d_o, lse, cu_seqlens, max_seqlen, scale, dq, dk, dv, workspace, *,
                    seqused=None, cu_seqlens_host=None, reuse_schedule=False, only=None, dropout=None):
    """Enqueue the backward pass on torch's current stream; fills dq, dk, dv.
    `only` = "dq" or "dkv" runs one of the two passes (see the header);
    `dropout` = (p, seed) selects fmha_varlen_bwd_dropout."""
    extra = {None: 0, "dq": FMHA_FLAG_BWD_ONLY_DQ, "dkv": FMHA_FLAG_BWD_ONLY_DKV}[only]
    p, keep = _params(q, cu_seqlens, max_seqlen, scale, workspace, seqused, cu_seqlens_host,
                      reuse_schedule, extra)
    p.q_stride, p.k_stride, p.v_stride, p.o_stride = map(_tok_stride, (q, k, v, o))
    p.do_stride, p.dq_stride, p.dk_stride, p.dv_stride = map(_tok_stride, (d_o, dq, dk, dv))
    ptrs = (q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
            dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _stream())
    if dropout is None:
        _check(lib().fmha_varlen_bwd(ctypes.byref(p), *ptrs))
    else:
        d = _dropout(dropout)
        _check(lib().fmha_varlen_bwd_dropout(ctypes.byref(p), ctypes.byref(d), *ptrs))
    del keep


def fmha_dropout_keep_mask(heads, cu_seqlens, max_seqlen, dropout, mask, workspace, *, orientation=0,
                           cu_seqlens_host=None):
    """Enqueue the kernel that writes the keep mask into `mask` (uint8 [heads, T, row_bytes])."""
    assert mask.dtype == torch.uint8 and mask.is_contiguous() and mask.dim() == 3 and mask.shape[0] == heads
    p = Params()
    p.batch = cu_seqlens.numel() - 1
    p.total_tokens, p.heads, p.head_dim = mask.shape[1], heads, 64
    p.max_seqlen = int(max_seqlen)
    p.dtype = FMHA_F16
    p.scale = 1.0
    p.cu_seqlens = cu_seqlens.data_ptr()
    keep = []
    if cu_seqlens_host is not None:
        h = cu_seqlens_host.to(dtype=torch.int32, device="cpu").contiguous()
        keep.append(h)
        p.cu_seqlens_host = h.data_ptr()
    p.workspace = workspace.data_ptr()
    p.workspace_bytes = workspace.numel() * workspace.element_size()
    d = _dropout(dropout)
    _check(lib().fmha_dropout_keep_mask(ctypes.byref(p), ctypes.byref(d), int(orientation),
                                        mask.shape[2], mask.data_ptr(), _stream()))
    del keep


def fmha_unpad_indices_host(input_mask):
    """input_mask: CPU int32 tensor [B, S].  Returns (nonzero_indices [n], inverse [B*S],
    cu_seqlens [B+1], max_seqlen) computed by the library's host routine."""
    m = input_mask.to(dtype=torch.int32, device="cpu").contiguous()
    nb, s = m.shape
    idx = torch.empty(nb * s, dtype=torch.int32)
    inv = torch.empty(nb * s, dtype=torch.int32)
    cu = torch.empty(nb + 1, dtype=torch.int32)
    mx = ctypes.c_int32(0)
    _check(lib().fmha_unpad_indices_host(m.data_ptr(), nb, s, idx.data_ptr(), inv.data_ptr(), cu.data_ptr(),
                                         ctypes.addressof(mx)))
    return idx[:int(cu[-1])], inv, cu, int(mx.value)


def fmha_unpad_indices(input_mask, nonzero_indices, inverse, cu_seqlens):
    """Device version: input_mask int32 [B, S] on the GPU; fills the three device arrays."""
    nb, s = input_mask.shape
    assert input_mask.dtype == torch.int32 and input_mask.is_cuda and input_mask.is_contiguous()
    assert nonzero_indices.numel() >= nb * s and cu_seqlens.numel() == nb + 1
    assert inverse is None or inverse.numel() == nb * s
    _check(lib().fmha_unpad_indices(input_mask.data_ptr(), nb, s, nonzero_indices.data_ptr(),
                                    None if inverse is None else inverse.data_ptr(),
                                    cu_seqlens.data_ptr(), _stream()))


def _rows(t):
    assert t.is_cuda and t.is_contiguous() and t.dim() >= 2
    return t.shape[0], (t.numel() // max(t.shape[0], 1)) * t.element_size()


def fmha_gather_rows(padded, nonzero_indices, n_rows, packed):
    """packed[j] = padded[nonzero_indices[j]] for j < n_rows[0] (a device int32)."""
    pr, rb = _rows(padded)
    kr, rb2 = _rows(packed)
    assert rb == rb2 or kr == 0 or pr == 0
    _check(lib().fmha_gather_rows(padded.data_ptr(), pr, nonzero_indices.data_ptr(), n_rows.data_ptr(),
                                  kr, rb if pr else rb2, packed.data_ptr(), _stream()))


def fmha_scatter_rows(packed, inverse, n_rows, padded):
    """padded[r] = packed[inverse[r]] where that is a valid packed row, zeros elsewhere."""
    kr, rb = _rows(packed)
    pr, rb2 = _rows(padded)
    assert rb == rb2 or kr == 0 or pr == 0
    _check(lib().fmha_scatter_rows(packed.data_ptr(), kr, inverse.data_ptr(), n_rows.data_ptr(),
                                   pr, rb2 if pr else rb, padded.data_ptr(), _stream()))


def _ln_params(t, eps, dropout, n_rows):
    assert t.dim() == 2 and t.is_contiguous() and t.is_cuda
    p = LnParams()
    p.rows, p.hidden = t.shape
    p.dtype = _dtype_code(t)
    p.eps = float(eps)
    if n_rows is not None:
        assert n_rows.dtype == torch.int32 and n_rows.is_cuda
        p.n_rows = n_rows.data_ptr()
    p.dropout = _dropout(dropout) if dropout is not None else Dropout(0.0, 0)
    return p


def fmha_dropout_add_ln_bwd_workspace_size(rows: int, hidden: int) -> int:
    return int(lib().fmha_dropout_add_ln_bwd_workspace_size(rows, hidden))


def fmha_dropout_add_ln_fwd(x, residual, gamma, beta, eps, y, z, mu, rstd, *, dropout=None, n_rows=None):
    """y = LayerNorm(dropout(x) + residual) on [rows, hidden] 16-bit tensors; fills y, z, mu, rstd."""
    p = _ln_params(x, eps, dropout, n_rows)
    for t in (residual, y, z):
        assert t.shape == x.shape and t.dtype == x.dtype and t.is_contiguous()
    for t in (gamma, beta, mu, rstd):
        assert t.dtype == torch.float32 and t.is_contiguous()
    _check(lib().fmha_dropout_add_ln_fwd(ctypes.byref(p), x.data_ptr(), residual.data_ptr(), gamma.data_ptr(),
                                         beta.data_ptr(), y.data_ptr(), z.data_ptr(), mu.data_ptr(),
                                         rstd.data_ptr(), _stream()))


def fmha_dropout_add_ln_bwd(dy, z, mu, rstd, gamma, eps, dx, dresidual, dgamma, dbeta, workspace, *,
                            dropout=None, n_rows=None):
    """Backward of fmha_dropout_add_ln_fwd; fills dx, dresidual (unless None), dgamma, dbeta."""
    p = _ln_params(dy, eps, dropout, n_rows)
    _check(lib().fmha_dropout_add_ln_bwd(ctypes.byref(p), dy.data_ptr(), z.data_ptr(), mu.data_ptr(),
                                         rstd.data_ptr(), gamma.data_ptr(), dx.data_ptr(),
                                         None if dresidual is None else dresidual.data_ptr(),
                                         dgamma.data_ptr(), dbeta.data_ptr(), workspace.data_ptr(),
                                         workspace.numel() * workspace.element_size(), _stream()))


def fmha_embedding_sort_workspace_size(rows: int, hidden: int) -> int:
    return int(lib().fmha_embedding_sort_workspace_size(rows, hidden))


def fmha_embedding_sort(indices, hidden, vocab, workspace, *, padding_idx=-1, n_rows=None):
    """Orders the token positions by index into `workspace` (uint8 device tensor of
    fmha_embedding_sort_workspace_size(rows, hidden) bytes) for fmha_embedding_bwd_sorted."""
    assert indices.dtype == torch.int32 and indices.is_cuda and indices.dim() == 1
    _check(lib().fmha_embedding_sort(indices.data_ptr(), None if n_rows is None else n_rows.data_ptr(),
                                     indices.numel(), int(hidden), int(vocab), int(padding_idx), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream()))


def fmha_embedding_bwd_sorted(dy, workspace, dw, *, zero_first=False):
    """dw[i] += sum of the rows dy[t] with indices[t] = i, in the order fmha_embedding_sort left in
    `workspace`: fp32 sums, one write per weight row, no atomics."""
    assert dy.dim() == 2 and dw.dim() == 2 and dy.is_contiguous() and dw.is_contiguous() and dy.dtype == dw.dtype
    _check(lib().fmha_embedding_bwd_sorted(dy.data_ptr(), workspace.data_ptr(),
                                           workspace.numel() * workspace.element_size(), dy.shape[0], dy.shape[1],
                                           dw.shape[0], _dtype_code(dy), FMHA_EMB_ZERO_FIRST if zero_first else 0,
                                           dw.data_ptr(), _stream()))


def fmha_embedding_bwd(dy, indices, dw, *, padding_idx=-1, n_rows=None, zero_first=False, plain_split=False,
                       no_die_split=False):
    """dw[indices[t]] += dy[t] with packed 16-bit atomic adds; dy [T, N], indices int32 [T], dw [V, N]."""
    assert dy.dim() == 2 and dw.dim() == 2 and dy.is_contiguous() and dw.is_contiguous() and dy.dtype == dw.dtype
    assert indices.dtype == torch.int32 and indices.is_cuda and indices.numel() == dy.shape[0]
    flags = ((FMHA_EMB_ZERO_FIRST if zero_first else 0) | (FMHA_EMB_PLAIN_SPLIT if plain_split else 0)
             | (FMHA_EMB_NO_DIE_SPLIT if no_die_split else 0))
    _check(lib().fmha_embedding_bwd(dy.data_ptr(), indices.data_ptr(), None if n_rows is None else n_rows.data_ptr(),
                                    dy.shape[0], dy.shape[1], dw.shape[0], int(padding_idx), _dtype_code(dy), flags,
                                    dw.data_ptr(), _stream()))
