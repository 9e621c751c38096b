"""Seeded synthetic inputs for packed variable-length attention.

This module only draws lengths and tensors and lays them out; it contains none
of the attention arithmetic, so both the CPU oracle's tests and the HIP path's
tests/bench can use it without sharing any of the method's code.

Layout follows the paper's unpadded storage (Section IV-A-1, "storage for unpad
computing"): the batch and sequence dimensions are merged, only valid tokens
are stored, and a prefix-sum array (`cu_seqlens`, the paper's batch_offset)
records where each sequence starts.

The five workloads stand in for the paper's MLPerf BERT (Wikipedia) batches,
which are not available: 56 sequences per GPU and max length 512 as in
Section V, with a large share of sequences at the maximum length as in the
paper's sequence-length statistics (Section III-C).
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 220808124
HEAD_DIM = 64


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    dtype: str          # "f16" or "bf16"
    max_seqlen: int
    seed: int
    backward: bool
    mixture: str        # description of the length distribution


WORKLOADS = {
    1: Workload("tiny_fwd", 4, 2, "f16", 128, BASE_SEED + 1, False,
                "fixed lengths 3,17,64,128"),
    2: Workload("bert_large_fwd", 56, 16, "f16", 512, BASE_SEED + 2, False,
                "30% U[1,128], 40% U[129,511], 30% =512"),
    3: Workload("bert_large_fwd_bwd", 56, 16, "f16", 512, BASE_SEED + 2, True,
                "30% U[1,128], 40% U[129,511], 30% =512"),
    4: Workload("skewed_fwd_bwd", 256, 16, "f16", 512, BASE_SEED + 4, True,
                "60% U[1,64], 25% U[65,256], 15% =512"),
    5: Workload("large_packed_fwd_bwd", 2048, 12, "bf16", 512, BASE_SEED + 5, True,
                "U[1,512]"),
}


def draw_lengths(cfg: int, rng: np.random.Generator) -> np.ndarray:
    """Sequence lengths of workload `cfg`, in pack order (unsorted)."""
    w = WORKLOADS[cfg]
    if cfg == 1:
        return np.array([3, 17, 64, 128], dtype=np.int32)
    u = rng.random(w.batch)
    out = np.empty(w.batch, dtype=np.int32)
    if cfg in (2, 3):
        a = rng.integers(1, 129, size=w.batch)
        b = rng.integers(129, 512, size=w.batch)
        out[:] = np.where(u < 0.3, a, np.where(u < 0.7, b, 512))
    elif cfg == 4:
        a = rng.integers(1, 65, size=w.batch)
        b = rng.integers(65, 257, size=w.batch)
        out[:] = np.where(u < 0.60, a, np.where(u < 0.85, b, 512))
    elif cfg == 5:
        out[:] = rng.integers(1, 513, size=w.batch)
    else:
        raise ValueError(cfg)
    return out


def cu_from_lengths(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    np.cumsum(np.asarray(lengths, dtype=np.int64), out=cu[1:])
    return cu


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    b = b + 0x7FFF + ((b >> 16) & 1)
    return (b >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def to_bits(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the 16-bit storage type; returns uint16 bit patterns."""
    if dtype == "f16":
        return x32.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x32)
    raise ValueError(dtype)


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored 16-bit values to float64."""
    if dtype == "f16":
        return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(bits).astype(np.float64)
    raise ValueError(dtype)


def normal_bits(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    return to_bits(rng.standard_normal(shape, dtype=np.float32), dtype)


def make_batch(lengths, heads: int, dtype: str, seed: int, backward: bool = True,
               scale: float = 0.125) -> dict:
    """Packed Q, K, V (and dO) as uint16 bit patterns of shape [T, heads, 64]."""
    lengths = np.asarray(lengths, dtype=np.int32)
    rng = np.random.default_rng(seed)
    t = int(lengths.sum())
    shape = (t, heads, HEAD_DIM)
    out = {
        "lengths": lengths, "cu_seqlens": cu_from_lengths(lengths),
        "batch": len(lengths), "heads": heads, "total_tokens": t,
        "max_seqlen": int(lengths.max()) if len(lengths) else 0,
        "dtype": dtype, "scale": float(scale),
        "q": normal_bits(rng, shape, dtype),
        "k": normal_bits(rng, shape, dtype),
        "v": normal_bits(rng, shape, dtype),
    }
    if backward:
        out["do"] = normal_bits(np.random.default_rng([seed, 1]), shape, dtype)
    return out


def make_workload(cfg: int, backward: bool | None = None) -> dict:
    """One of the five named workloads, fully materialised on the host."""
    w = WORKLOADS[cfg]
    rng = np.random.default_rng(w.seed)
    lengths = draw_lengths(cfg, rng)
    bwd = w.backward if backward is None else backward
    # tensors come from a generator seeded apart from the length draw so that
    # workloads 2 and 3 share lengths and Q, K, V exactly
    b = make_batch(lengths, w.heads, w.dtype, w.seed + 1000, backward=bwd)
    b["name"] = w.name
    b["max_seqlen"] = w.max_seqlen
    return b


def pad_batch(batch: dict, max_seqlen: int) -> dict:
    """Same data in the padded layout: sequence i occupies rows
    [i*max_seqlen, (i+1)*max_seqlen), rows past its length are zero.  `seqused`
    carries the valid length so that keys past it can be masked."""
    lengths = batch["lengths"]
    nb, h = len(lengths), batch["heads"]
    cu = batch["cu_seqlens"]
    out = dict(batch)
    out["cu_seqlens"] = (np.arange(nb + 1, dtype=np.int64) * max_seqlen).astype(np.int32)
    out["seqused"] = lengths.astype(np.int32).copy()
    out["total_tokens"] = nb * max_seqlen
    out["max_seqlen"] = max_seqlen
    for name in ("q", "k", "v", "do"):
        if name not in batch:
            continue
        p = np.zeros((nb * max_seqlen, h, HEAD_DIM), dtype=np.uint16)
        for i in range(nb):
            p[i * max_seqlen:i * max_seqlen + lengths[i]] = batch[name][cu[i]:cu[i + 1]]
        out[name] = p
    return out


def valid_row_index(lengths, max_seqlen: int) -> np.ndarray:
    """Row numbers, in the padded layout, of the valid tokens in pack order."""
    return np.concatenate([i * max_seqlen + np.arange(l) for i, l in enumerate(lengths)]
                          or [np.zeros(0, dtype=np.int64)]).astype(np.int64)


def useful_flops(lengths, heads: int, backward: bool) -> float:
    """4*sum(L^2)*H*d forward, plus 10*sum(L^2)*H*d backward (five contractions)."""
    s2 = float((np.asarray(lengths, dtype=np.float64) ** 2).sum())
    return (14.0 if backward else 4.0) * s2 * heads * HEAD_DIM


def zipf_token_ids(n: int, vocab: int, seed: int, exponent: float = 1.0) -> np.ndarray:
    """n token ids in [0, vocab) whose frequencies follow a Zipf law (rank r has weight
    r**-exponent), the ranks assigned to ids by a seeded permutation: a stand-in for the
    word-piece ids of the paper's Wikipedia batches (a few very frequent ids, a long tail)."""
    rng = np.random.default_rng(seed)
    w = np.arange(1, vocab + 1, dtype=np.float64) ** -exponent
    cdf = np.cumsum(w / w.sum())
    ranks = np.minimum(np.searchsorted(cdf, rng.random(n)), vocab - 1)
    return rng.permutation(vocab)[ranks].astype(np.int32)
