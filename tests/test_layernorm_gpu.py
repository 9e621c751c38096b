"""Dropout + Add + LayerNorm on the GPU against oracle/layernorm.py, through the C ABI.

Tolerances (derived from the arithmetic: fp32 math, 16-bit stores; the backward works
from the stored 16-bit z): y within 2e-3 + one 16-bit ulp of the reference value; mu within
1e-5 * max|z| ; rstd within 1e-4 relative; dx, dresidual per tensor within 1e-2 of the
largest reference magnitude (the attention path's gradient bar); dgamma, dbeta (fp32
sums over rows of 16-bit-accurate terms) within 1e-2 of the largest reference magnitude.
"""
import numpy as np
import pytest
import torch

from oracle import dropout_mask as dm
from oracle import layernorm as ln
from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl
from gpu_util import TORCH_DT, to_dev, to_f64, ulp_half

pytestmark = pytest.mark.gpu


def make(rows, hidden, dtype, seed):
    rng = np.random.default_rng(seed)
    bits = lambda a: wl.to_bits(a.astype(np.float32), dtype)
    x, r, dy = (bits(rng.standard_normal((rows, hidden))) for _ in range(3))
    gamma = (1.0 + 0.2 * rng.standard_normal(hidden)).astype(np.float32)
    beta = (0.5 * rng.standard_normal(hidden)).astype(np.float32)
    return x, r, dy, gamma, beta


class Run:
    def __init__(self, rows, hidden, dtype, seed, p=0.0, dseed=0, eps=1e-5, cap=None, with_dr=True):
        self.rows, self.hidden, self.dtype, self.p, self.dseed, self.eps = rows, hidden, dtype, p, dseed, eps
        cap = rows if cap is None else cap
        self.x, self.r, self.dy, self.gamma, self.beta = make(cap, hidden, dtype, seed)
        d = lambda b: to_dev(b, dtype)
        tdt = TORCH_DT[dtype]
        self.dx_, self.dr_, self.ddy = d(self.x), d(self.r), d(self.dy)
        self.dg, self.db = torch.from_numpy(self.gamma).cuda(), torch.from_numpy(self.beta).cuda()
        nan16 = lambda: torch.full((cap, hidden), float("nan"), dtype=tdt, device="cuda")
        self.y, self.z, self.gx, self.gr = nan16(), nan16(), nan16(), (nan16() if with_dr else None)
        self.mu = torch.full((cap,), float("nan"), dtype=torch.float32, device="cuda")
        self.rstd = torch.full((cap,), float("nan"), dtype=torch.float32, device="cuda")
        self.ggamma = torch.full((hidden,), float("nan"), dtype=torch.float32, device="cuda")
        self.gbeta = torch.full((hidden,), float("nan"), dtype=torch.float32, device="cuda")
        self.n_rows = torch.tensor([rows], dtype=torch.int32, device="cuda") if cap != rows else None
        ws = max(fmha.fmha_dropout_add_ln_bwd_workspace_size(cap, hidden), 16)
        self.ws = torch.empty(ws, dtype=torch.uint8, device="cuda")
        drop = (p, dseed) if p else None
        fmha.fmha_dropout_add_ln_fwd(self.dx_, self.dr_, self.dg, self.db, eps, self.y, self.z, self.mu, self.rstd,
                                     dropout=drop, n_rows=self.n_rows)
        fmha.fmha_dropout_add_ln_bwd(self.ddy, self.z, self.mu, self.rstd, self.dg, eps, self.gx, self.gr,
                                     self.ggamma, self.gbeta, self.ws, dropout=drop, n_rows=self.n_rows)
        torch.cuda.synchronize()

    def check(self):
        n, dt = self.rows, self.dtype
        f = lambda b: wl.bits_to_f64(b[:n], dt)
        x, r, dy = f(self.x), f(self.r), f(self.dy)
        mask = ln.ln_keep_mask(n, self.hidden, self.p, self.dseed) if self.p else None
        c = dm.keep_scale(self.p) if self.p else 1.0
        y, z, mu, rstd = ln.fwd(x, r, self.gamma, self.beta, self.eps, mask, c)
        dx, dr, dgamma, dbeta = ln.bwd(dy, x, r, self.gamma, self.eps, mask, c)
        if n:
            gy, gz = to_f64(self.y[:n]), to_f64(self.z[:n])
            assert not np.isnan(gy).any() and not np.isnan(gz).any()
            assert (np.abs(gy - y) <= 2e-3 + 2 * ulp_half(y, dt)).all(), f"y: {np.abs(gy - y).max():.3e}"
            assert (np.abs(gz - z) <= 1e-6 + ulp_half(z, dt) * 1.01).all(), f"z: {np.abs(gz - z).max():.3e}"
            assert np.abs(to_f64(self.mu[:n]) - mu).max() <= 1e-5 * max(1.0, np.abs(z).max())
            assert (np.abs(to_f64(self.rstd[:n]) - rstd) <= 1e-4 * rstd).all()
            for name, got, want in (("dx", self.gx, dx), ("dr", self.gr, dr)):
                if got is None:
                    continue
                g = to_f64(got[:n])
                assert not np.isnan(g).any(), name
                rel = np.abs(g - want).max() / max(np.abs(want).max(), 1e-3)
                assert rel <= 1e-2, f"{name}: {rel:.3e}"
        for name, got, want in (("dgamma", self.ggamma, dgamma), ("dbeta", self.gbeta, dbeta)):
            g = to_f64(got)
            assert not np.isnan(g).any(), name
            rel = np.abs(g - want).max() / max(np.abs(want).max(), 1e-3)
            assert rel <= 1e-2, f"{name}: {rel:.3e}"
        return self


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("rows,hidden", [(1, 16), (3, 48), (5, 768), (70, 1024), (33, 1040), (9, 2048), (7, 3072), (4, 4096), (0, 64)])
def test_layernorm_no_dropout(rows, hidden, dtype):
    Run(rows, hidden, dtype, seed=rows * 131 + hidden).check()


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("rows,hidden,p", [(2, 16, 0.5), (37, 768, 0.1), (130, 1024, 0.1), (6, 2064, 0.3), (5, 4096, 0.1)])
def test_layernorm_with_dropout(rows, hidden, p, dtype):
    Run(rows, hidden, dtype, seed=rows + hidden, p=p, dseed=0x1234567811223344 + rows).check()


def test_layernorm_many_rows_bert_large_shape():
    """Workload 3's token count x BERT-large hidden size: every persistent wavefront takes
    several rows and the column sums span hundreds of workgroups' partial results."""
    t = int(wl.make_workload(3)["total_tokens"])
    Run(t, 1024, "f16", seed=3, p=0.1, dseed=77).check()


def test_device_row_count_leaves_the_tail_alone():
    r = Run(50, 1024, "f16", seed=9, p=0.1, dseed=5, cap=80).check()
    for t in (r.y, r.z, r.gx, r.gr):
        assert torch.isnan(t[50:].float()).all(), "rows beyond n_rows were written"
    assert torch.isnan(r.mu[50:]).all() and torch.isnan(r.rstd[50:]).all()


def test_null_dresidual_and_reproducibility():
    a = Run(300, 768, "bf16", seed=4, with_dr=False).check()
    b = Run(300, 768, "bf16", seed=4).check()
    assert torch.equal(a.gx, b.gx) and torch.equal(b.gx, b.gr)      # no dropout: dx = dresidual
    assert torch.equal(a.ggamma, b.ggamma) and torch.equal(a.gbeta, b.gbeta)


def test_layernorm_argument_errors():
    x = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    g = torch.zeros(64, dtype=torch.float32, device="cuda")
    s = torch.zeros(4, dtype=torch.float32, device="cuda")
    with pytest.raises(fmha.FmhaError) as e:
        fmha.fmha_dropout_add_ln_fwd(x[:, :40].contiguous(), x[:, :40].contiguous(), g, g, 1e-5,
                                     x[:, :40].contiguous(), x[:, :40].contiguous(), s, s)
    assert e.value.code == fmha.FMHA_ERR_INVALID_ARG and "multiple of 16" in str(e.value)
    with pytest.raises(fmha.FmhaError) as e:
        fmha.fmha_dropout_add_ln_fwd(x, x, g, g, 1e-5, x, x, s, s, dropout=(1.5, 1))
    assert e.value.code == fmha.FMHA_ERR_INVALID_ARG
    ws = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(fmha.FmhaError) as e:
        fmha.fmha_dropout_add_ln_bwd(x, x, s, s, g, 1e-5, x, None, g, g, ws)
    assert e.value.code == fmha.FMHA_ERR_WORKSPACE
    assert fmha.fmha_dropout_add_ln_bwd_workspace_size(4, 40) == 0


def test_layernorm_half_a_million_rows_sampled():
    """Workload 5's shape (527 340 rows x 768, bf16, p = 0.1): every persistent wavefront takes
    dozens of rows.  Row ranges at the start, in the middle and at the end are checked against
    the oracle (all per-row results).  Of the column sums only dbeta (the plain column sum of dy)
    has a cheap exact reference at this size; dgamma is checked against the oracle at 15 769
    rows above."""
    rows, hidden, p, seed = 527340, 768, 0.1, 99
    g = torch.Generator(device="cuda").manual_seed(1)
    rnd = lambda: torch.randn((rows, hidden), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    x, r, dy = rnd(), rnd(), rnd()
    gamma = 1 + 0.2 * torch.randn(hidden, generator=g, device="cuda")
    beta = 0.5 * torch.randn(hidden, generator=g, device="cuda")
    y, z, dx, dr = (torch.full_like(x, float("nan")) for _ in range(4))
    mu, rstd = (torch.full((rows,), float("nan"), device="cuda") for _ in range(2))
    dgamma, dbeta = (torch.full((hidden,), float("nan"), device="cuda") for _ in range(2))
    ws = torch.empty(fmha.fmha_dropout_add_ln_bwd_workspace_size(rows, hidden), dtype=torch.uint8, device="cuda")
    fmha.fmha_dropout_add_ln_fwd(x, r, gamma, beta, 1e-5, y, z, mu, rstd, dropout=(p, seed))
    fmha.fmha_dropout_add_ln_bwd(dy, z, mu, rstd, gamma, 1e-5, dx, dr, dgamma, dbeta, ws, dropout=(p, seed))
    torch.cuda.synchronize()
    for t in (y, z, dx, dr, mu, rstd, dgamma, dbeta):
        assert not torch.isnan(t.float()).any(), "rows left unwritten"
    c = dm.keep_scale(p)
    gm, bt = gamma.double().cpu().numpy(), beta.double().cpu().numpy()
    for first in (0, rows // 2 - 7, rows - 48):
        sl = slice(first, first + 48)
        mask = ln.ln_keep_mask(48, hidden, p, seed, first_row=first)
        xs, rs, dys = (to_f64(t[sl]) for t in (x, r, dy))
        y_ref, z_ref, mu_ref, rstd_ref = ln.fwd(xs, rs, gm, bt, 1e-5, mask, c)
        dx_ref, dr_ref, _, _ = ln.bwd(dys, xs, rs, gm, 1e-5, mask, c)
        assert (np.abs(to_f64(y[sl]) - y_ref) <= 2e-3 + 2 * ulp_half(y_ref, "bf16")).all()
        assert (np.abs(to_f64(z[sl]) - z_ref) <= 1e-6 + ulp_half(z_ref, "bf16") * 1.01).all()
        assert (np.abs(to_f64(rstd[sl]) - rstd_ref) <= 1e-4 * rstd_ref).all()
        for got, want in ((dx, dx_ref), (dr, dr_ref)):
            assert np.abs(to_f64(got[sl]) - want).max() <= 1e-2 * max(np.abs(want).max(), 1e-3)
    # dbeta is the plain column sum of dy: an exact reference is cheap
    want = dy.double().sum(dim=0).cpu().numpy()
    assert np.abs(to_f64(dbeta) - want).max() <= 1e-3 * np.abs(want).max() + 1e-2
