"""Helpers shared by the GPU parity tests: move a host batch (uint16 bit
patterns) to the device, run the HIP path through the C ABI, bring results
back as float64."""
import numpy as np
import torch

from paper_2208_08124_amd import fmha
from paper_2208_08124_amd import workloads as wl

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def to_dev(bits: np.ndarray, dtype: str) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TORCH_DT[dtype])


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


class DeviceBatch:
    def __init__(self, b: dict, need_bwd: bool):
        self.b = b
        dt = b["dtype"]
        self.q, self.k, self.v = (to_dev(b[n], dt) for n in ("q", "k", "v"))
        self.do = to_dev(b["do"], dt) if need_bwd else None
        self.cu = torch.from_numpy(b["cu_seqlens"]).cuda()
        self.seqused = torch.from_numpy(b["seqused"]).cuda() if "seqused" in b else None
        t, h = b["total_tokens"], b["heads"]
        self.o = torch.full_like(self.q, float("nan"))
        self.lse = torch.full((h, t), float("nan"), dtype=torch.float32, device="cuda")
        self.ws = fmha.alloc_workspace(b["batch"], t, h, need_bwd)
        if need_bwd:
            self.dq, self.dk, self.dv = (torch.full_like(self.q, float("nan")) for _ in range(3))

    def fwd(self, **kw):
        b = self.b
        fmha.fmha_varlen_fwd(self.q, self.k, self.v, self.cu, b["max_seqlen"], b["scale"],
                             self.o, self.lse, self.ws, seqused=self.seqused, **kw)

    def bwd(self, **kw):
        b = self.b
        fmha.fmha_varlen_bwd(self.q, self.k, self.v, self.o, self.do, self.lse, self.cu,
                             b["max_seqlen"], b["scale"], self.dq, self.dk, self.dv, self.ws,
                             seqused=self.seqused, **kw)


def oracle_inputs(b: dict):
    dt = b["dtype"]
    return {n: wl.bits_to_f64(b[n], dt) for n in ("q", "k", "v", "do") if n in b}


def ulp_half(x: np.ndarray, dtype: str) -> np.ndarray:
    """Half a unit in the last place of the 16-bit type at |x| (normal range)."""
    mant = 10 if dtype == "f16" else 7
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -14)))
    return 0.5 * 2.0 ** (e - mant)
