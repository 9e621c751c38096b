"""Host-side checks of the C-ABI library that need no GPU: the library loads,
exports every function the header declares, sizes workspaces, and rejects bad
arguments with the documented codes before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2208_08124_amd", "libfmha_varlen.so")
HEADER = os.path.join(ROOT, "include", "fmha_varlen.h")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="library not built (run __graft_entry__.build())")


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(fmha_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported():
    lib = ctypes.CDLL(LIB)
    names = declared_functions()
    assert {"fmha_varlen_fwd", "fmha_varlen_bwd", "fmha_varlen_workspace_size",
            "fmha_varlen_schedule_info", "fmha_last_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_mirrors_the_header():
    from paper_2208_08124_amd import fmha
    assert set(fmha.EXPORTS) == set(declared_functions())
    # struct layout: 8 x 4-byte fields, 8 x int64 strides, 4 pointers, size_t
    assert ctypes.sizeof(fmha.Params) == 8 * 4 + 8 * 8 + 4 * 8 + 8
    hdr = open(HEADER).read()
    for flag, val in (("FMHA_FLAG_REUSE_SCHEDULE", fmha.FMHA_FLAG_REUSE_SCHEDULE),
                      ("FMHA_FLAG_BWD_ONLY_DQ", fmha.FMHA_FLAG_BWD_ONLY_DQ),
                      ("FMHA_FLAG_BWD_ONLY_DKV", fmha.FMHA_FLAG_BWD_ONLY_DKV)):
        assert re.search(r"#define\s+%s\s+%du" % (flag, val), hdr)


def test_workspace_size_arithmetic():
    from paper_2208_08124_amd import fmha
    f = fmha.fmha_varlen_workspace_size
    assert f(-1, 10, 2, False) == 0 and f(1, -1, 2, False) == 0 and f(1, 1, 0, True) == 0
    small, big = f(4, 212, 2, False), f(4, 212, 2, True)
    # header line, 2 KB of hand-out counters, then the 16-byte tile records
    assert small >= 256 + 2048 + 16 * (212 // 128 + 4) and small % 256 == 0
    assert big >= small + 2 * 4 * (212 * 2 + 1) and big % 256 == 0
    cap, c_off, l_off = fmha.fmha_varlen_schedule_info(4, 212)
    assert cap == 212 // 128 + 4 and c_off == 0 and l_off == 256 + 2048
    # monotone in every size
    assert f(5, 212, 2, True) >= big and f(4, 300, 2, True) >= big and f(4, 212, 3, True) >= big


class Fake:
    """Aligned, non-null host addresses standing in for device pointers: every case below
    fails validation, which reads host memory only, so nothing is ever dereferenced."""
    def __init__(self):
        self.buf = np.zeros(4096, dtype=np.uint8)
        base = self.buf.ctypes.data
        self.p = (base + 255) // 256 * 256


def call_fwd(fmha, **over):
    fk = Fake()
    p = fmha.Params()
    p.batch, p.total_tokens, p.heads, p.head_dim, p.max_seqlen = 2, 16, 2, 64, 8
    p.dtype, p.flags, p.scale = fmha.FMHA_F16, 0, 0.125
    p.cu_seqlens = fk.p
    p.workspace, p.workspace_bytes = fk.p, 1 << 20
    ptrs = dict(q=fk.p, k=fk.p, v=fk.p, o=fk.p, lse=fk.p)
    keep = [fk]
    for k_, v_ in over.items():
        if k_ in ptrs:
            ptrs[k_] = v_
        elif k_ == "cu_host":
            arr = np.asarray(v_, dtype=np.int32)
            keep.append(arr)
            p.cu_seqlens_host = arr.ctypes.data
        else:
            setattr(p, k_, v_)
    rc = fmha.lib().fmha_varlen_fwd(ctypes.byref(p), ptrs["q"], ptrs["k"], ptrs["v"], ptrs["o"],
                                    ptrs["lse"], None)
    return rc, fmha.last_error()


def test_forward_rejects_bad_arguments_without_a_device():
    from paper_2208_08124_amd import fmha
    INV, UNS, WS = fmha.FMHA_ERR_INVALID_ARG, fmha.FMHA_ERR_UNSUPPORTED, fmha.FMHA_ERR_WORKSPACE
    cases = [
        (dict(head_dim=128), UNS, "head_dim"),
        (dict(dtype=7), UNS, "dtype"),
        (dict(batch=-1), INV, "batch"),
        (dict(total_tokens=-5), INV, "total_tokens"),
        (dict(heads=0), INV, "heads"),
        (dict(scale=float("nan")), INV, "scale"),
        (dict(scale=float("inf")), INV, "scale"),
        (dict(cu_seqlens=0), INV, "cu_seqlens"),
        (dict(q=0), INV, "q is null"),
        (dict(o=Fake().p + 2), INV, "aligned"),
        (dict(q_stride=64), INV, "q_stride"),        # smaller than heads*64
        (dict(v_stride=132), INV, "v_stride"),       # not a multiple of 8
        (dict(k_stride=(1 << 24) + 8), INV, "2^24"),
        (dict(workspace=0), WS, "workspace"),
        (dict(workspace_bytes=64), WS, "workspace"),
        (dict(cu_host=[1, 8, 16]), INV, "expected 0"),
        (dict(cu_host=[0, 8, 7]), INV, "decreases"),
        (dict(cu_host=[0, 8, 15]), INV, "total_tokens"),
        (dict(cu_host=[0, 4, 16]), INV, "max_seqlen"),
    ]
    for over, code, frag in cases:
        rc, msg = call_fwd(fmha, **over)
        assert rc == code, (over, rc, msg)
        assert frag in msg, (over, msg)
    rc = fmha.lib().fmha_varlen_fwd(None, None, None, None, None, None, None)
    assert rc == INV


def test_backward_rejects_conflicting_pass_flags():
    from paper_2208_08124_amd import fmha
    fk = Fake()
    p = fmha.Params()
    p.batch, p.total_tokens, p.heads, p.head_dim = 1, 8, 1, 64
    p.dtype, p.scale = fmha.FMHA_BF16, 1.0
    p.flags = fmha.FMHA_FLAG_BWD_ONLY_DQ | fmha.FMHA_FLAG_BWD_ONLY_DKV
    p.cu_seqlens, p.workspace, p.workspace_bytes = fk.p, fk.p, 1 << 20
    a = [fk.p] * 10
    rc = fmha.lib().fmha_varlen_bwd(ctypes.byref(p), *a[:9], None)
    assert rc == fmha.FMHA_ERR_INVALID_ARG and "exclude" in fmha.last_error()


def test_static_forward_rejects_oversize_batches_on_the_host():
    """The size check of the allocation-free forward precedes every device call."""
    from paper_2208_08124_amd import fmha
    fk = Fake()
    limit = fmha.lib().fmha_varlen_static_scratch_bytes()
    assert limit == 1 << 20
    p = fmha.Params()
    p.batch, p.total_tokens, p.heads, p.head_dim, p.max_seqlen = 70000, 70000, 1, 64, 1
    p.dtype, p.scale, p.cu_seqlens = fmha.FMHA_F16, 0.125, fk.p
    assert fmha.fmha_varlen_workspace_size(p.batch, p.total_tokens, p.heads, False) > limit
    rc = fmha.lib().fmha_varlen_fwd_static(ctypes.byref(p), fk.p, fk.p, fk.p, fk.p, fk.p, None)
    assert rc == fmha.FMHA_ERR_WORKSPACE and "built-in scratch" in fmha.last_error()
    assert fmha.lib().fmha_varlen_fwd_static(None, fk.p, fk.p, fk.p, fk.p, fk.p, None) == fmha.FMHA_ERR_INVALID_ARG


def test_struct_layouts_against_the_c_compiler(tmp_path):
    """sizeof / offsetof of every struct in the header as gcc sees them, against the ctypes mirrors."""
    import subprocess
    from paper_2208_08124_amd import fmha
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "%s"\n'
                   'int main(void) {\n'
                   '  printf("%%zu %%zu %%zu\\n", sizeof(fmha_varlen_params_t), offsetof(fmha_varlen_params_t, cu_seqlens), offsetof(fmha_varlen_params_t, workspace_bytes));\n'
                   '  printf("%%zu %%zu\\n", sizeof(fmha_dropout_t), offsetof(fmha_dropout_t, seed));\n'
                   '  printf("%%zu %%zu %%zu %%zu\\n", sizeof(fmha_ln_params_t), offsetof(fmha_ln_params_t, eps), offsetof(fmha_ln_params_t, n_rows), offsetof(fmha_ln_params_t, dropout));\n'
                   '  return 0;\n}\n' % HEADER)
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Werror", "-o", str(exe), str(src)])
    rows = [[int(x) for x in l.split()] for l in subprocess.check_output([str(exe)]).decode().splitlines()]
    P, D, L = fmha.Params, fmha.Dropout, fmha.LnParams
    assert rows[0] == [ctypes.sizeof(P), P.cu_seqlens.offset, P.workspace_bytes.offset]
    assert rows[1] == [ctypes.sizeof(D), D.seed.offset]
    assert rows[2] == [ctypes.sizeof(L), L.eps.offset, L.n_rows.offset, L.dropout.offset]


def test_dropout_layernorm_embedding_reject_bad_arguments_without_a_device():
    from paper_2208_08124_amd import fmha
    lib, fk = fmha.lib(), Fake()
    INV, UNS, WS = fmha.FMHA_ERR_INVALID_ARG, fmha.FMHA_ERR_UNSUPPORTED, fmha.FMHA_ERR_WORKSPACE
    # dropout: null struct and p outside [0, 1)
    p = fmha.Params()
    p.batch, p.total_tokens, p.heads, p.head_dim = 1, 8, 1, 64
    p.dtype, p.scale = fmha.FMHA_F16, 1.0
    p.cu_seqlens, p.workspace, p.workspace_bytes = fk.p, fk.p, 1 << 20
    six = [fk.p] * 5 + [None]
    assert lib.fmha_varlen_fwd_dropout(ctypes.byref(p), None, *six) == INV and "dropout is null" in fmha.last_error()
    for bad in (1.0, -0.5, float("nan")):
        d = fmha.Dropout(bad, 1)
        assert lib.fmha_varlen_fwd_dropout(ctypes.byref(p), ctypes.byref(d), *six) == INV
        assert lib.fmha_varlen_bwd_dropout(ctypes.byref(p), ctypes.byref(d), *([fk.p] * 9), None) == INV
    d = fmha.Dropout(0.1, 1)
    assert lib.fmha_dropout_keep_mask(ctypes.byref(p), ctypes.byref(d), 2, 64, fk.p, None) == INV
    assert lib.fmha_dropout_keep_mask(ctypes.byref(p), ctypes.byref(d), 0, 0, fk.p, None) == INV
    # LayerNorm
    lp = fmha.LnParams()
    lp.rows, lp.hidden, lp.dtype, lp.eps = 4, 64, fmha.FMHA_F16, 1e-5
    nine = [fk.p] * 8 + [None]
    for field, val, code, frag in (("hidden", 40, INV, "multiple of 16"), ("hidden", 8192, UNS, "4096"),
                                   ("dtype", 9, UNS, "dtype"), ("rows", -1, INV, "rows"),
                                   ("eps", -1.0, INV, "eps")):
        q = fmha.LnParams.from_buffer_copy(lp)
        setattr(q, field, val)
        assert lib.fmha_dropout_add_ln_fwd(ctypes.byref(q), *nine) == code, field
        assert frag in fmha.last_error(), (field, fmha.last_error())
    assert lib.fmha_dropout_add_ln_fwd(None, *nine) == INV
    assert lib.fmha_dropout_add_ln_fwd(ctypes.byref(lp), None, *nine[1:]) == INV and "x is null" in fmha.last_error()
    assert lib.fmha_dropout_add_ln_bwd(ctypes.byref(lp), *([fk.p] * 9), None, 0, None) == WS
    assert fmha.fmha_dropout_add_ln_bwd_workspace_size(15769, 1024) == 256 * 2 * 1024 * 4
    assert fmha.fmha_dropout_add_ln_bwd_workspace_size(10, 1024) == 1 * 2 * 1024 * 4
    # embedding
    e = lib.fmha_embedding_bwd
    assert e(fk.p, fk.p, None, 4, 64, 10, -1, 5, 0, fk.p, None) == UNS
    assert e(fk.p, fk.p, None, 4, 60, 10, -1, 0, 0, fk.p, None) == INV and "multiple of 8" in fmha.last_error()
    assert e(fk.p, fk.p, None, 4, 64, 0, -1, 0, 0, fk.p, None) == INV
    assert e(None, fk.p, None, 4, 64, 10, -1, 0, 0, fk.p, None) == INV
    assert e(fk.p, fk.p, None, 4, 64, 10, -1, 0, 0, None, None) == INV


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
