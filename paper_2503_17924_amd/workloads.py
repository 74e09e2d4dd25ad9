"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This module draws numbers and nothing else: document-length lists shaped like
the long-context training mixes the paper describes (Section 2.2: a heavily
skewed length distribution, most documents short, the longest as long as the
context window), and bf16 tensors with i.i.d. N(0,1) entries.  It contains
none of the method's arithmetic (no attention, no sharding, no packing) and it
imports neither the oracle nor the HIP binding, so both sides can read the same
arrays without sharing any code of the method itself.

bf16 values travel as numpy uint16 bit patterns (numpy has no bf16 dtype).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np


# ----------------------------------------------------------------------------
# bf16 <-> float helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + rounding) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    """i.i.d. N(0,1) drawn in float32 and rounded to bf16 bits."""
    return f32_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


# ----------------------------------------------------------------------------
# document-length recipes
# ----------------------------------------------------------------------------
def uniform_docs_until_overflow(seed: int, total: int, lo: int, hi: int) -> np.ndarray:
    """Lengths uniform-int in [lo, hi]; the draw that would overflow `total` is
    discarded and the last document takes whatever is left (it may be < lo)."""
    rng = np.random.default_rng(seed)
    out, used = [], 0
    while True:
        d = int(rng.integers(lo, hi, endpoint=True))
        if used + d > total:
            break
        out.append(d)
        used += d
        if used == total:
            break
    if used < total:
        out.append(total - used)
    return np.asarray(out, dtype=np.int32)


def _mixture_draw(rng: np.random.Generator, tail_lo: int, tail_hi: int) -> int:
    """One document length from the long-tailed mix: 90 % log-normal body
    (median 1024 tokens, sigma 1.0, clipped to [16, 8192]), 10 % uniform tail."""
    u = rng.random()
    if u < 0.9:
        d = int(np.rint(rng.lognormal(mean=math.log(1024.0), sigma=1.0)))
        return min(max(d, 16), 8192)
    return int(rng.integers(tail_lo, tail_hi, endpoint=True))


def mixture_docs_fill(seed: int, total: int, tail_lo: int, tail_hi: int) -> np.ndarray:
    """Mixture lengths until the packed sequence is full; the document that
    crosses the end is truncated there (the paper's dataloader truncates long
    documents at the tail of the context window, Section 2.2)."""
    rng = np.random.default_rng(seed)
    out, used = [], 0
    while used < total:
        d = min(_mixture_draw(rng, tail_lo, tail_hi), total - used)
        out.append(d)
        used += d
    return np.asarray(out, dtype=np.int32)


def mixture_pool(seed: int, n_docs: int, tail_lo: int, tail_hi: int) -> np.ndarray:
    """A pool of n_docs mixture lengths in arrival order (no packing)."""
    rng = np.random.default_rng(seed)
    return np.asarray([_mixture_draw(rng, tail_lo, tail_hi) for _ in range(n_docs)], dtype=np.int32)


def straggler_docs(seed: int, total: int, long_len: int, lo: int, hi: int) -> np.ndarray:
    """One long document followed by tiny documents (uniform-int in [lo, hi])
    that fill the rest of the sequence; the last one is truncated."""
    rng = np.random.default_rng(seed)
    out, used = [long_len], long_len
    while used < total:
        d = min(int(rng.integers(lo, hi, endpoint=True)), total - used)
        out.append(d)
        used += d
    return np.asarray(out, dtype=np.int32)


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    doc_len: np.ndarray            # int32 [n_docs] (packed sequence) or a pool
    total_tokens: int
    hq: int
    hkv: int
    head_dim: int
    scale: float
    cp: int
    backward: bool
    tensor_seed: int
    extra: dict = field(default_factory=dict)

    def tensors(self, names=("q", "k", "v", "do"), total_tokens: int | None = None):
        """bf16 bit tensors for the full packed sequence, drawn in the fixed
        order Q, K, V, dO from default_rng(tensor_seed); Q and dO are
        [T, Hq, D], K and V are [T, Hkv, D]."""
        t = self.total_tokens if total_tokens is None else total_tokens
        rng = np.random.default_rng(self.tensor_seed)
        shapes = {"q": (t, self.hq, self.head_dim), "k": (t, self.hkv, self.head_dim),
                  "v": (t, self.hkv, self.head_dim), "do": (t, self.hq, self.head_dim)}
        out = {}
        for nm in ("q", "k", "v", "do"):
            arr = normal_bf16(rng, shapes[nm])
            if nm in names:
                out[nm] = arr
        return out


def config(idx: int) -> Workload:
    """The benchmark configurations, numbered as in the baseline description."""
    if idx == 0:
        return Workload("c0_4k_fwd_cp2", uniform_docs_until_overflow(0, 4096, 64, 1536), 4096,
                        hq=4, hkv=4, head_dim=64, scale=0.125, cp=2, backward=False, tensor_seed=1000)
    if idx == 1:
        return Workload("c1_32k_gqa_cp1", mixture_docs_fill(1, 32768, 8192, 32768), 32768,
                        hq=32, hkv=8, head_dim=128, scale=1.0 / math.sqrt(128.0), cp=1,
                        backward=True, tensor_seed=1001)
    if idx == 2:
        return Workload("c2_128k_cp8", mixture_docs_fill(2, 131072, 16384, 131072), 131072,
                        hq=8, hkv=1, head_dim=128, scale=1.0 / math.sqrt(128.0), cp=8,
                        backward=True, tensor_seed=1002)
    if idx == 3:
        return Workload("c3_pack_pool", mixture_pool(3, 2000, 8192, 131072), 131072,
                        hq=8, hkv=1, head_dim=128, scale=1.0 / math.sqrt(128.0), cp=1,
                        backward=True, tensor_seed=1003,
                        extra={"n_microbatch": 8, "l_max": 131072})
    if idx == 4:
        return Workload("c4_straggler", straggler_docs(4, 131072, 98304, 1, 64), 131072,
                        hq=16, hkv=2, head_dim=128, scale=1.0 / math.sqrt(128.0), cp=4,
                        backward=True, tensor_seed=1004)
    if idx == 5:
        # a second context window: the 64K setting of the paper's evaluation (Section 6.1, model and
        # parallelism table), one TP=4 share of a 7B-class layer (multi-head attention), CP=2
        return Workload("c5_64k_mha_cp2", mixture_docs_fill(5, 65536, 8192, 65536), 65536,
                        hq=8, hkv=8, head_dim=128, scale=1.0 / math.sqrt(128.0), cp=2,
                        backward=True, tensor_seed=1005)
    raise ValueError(f"no config {idx}")


def small_case(seed: int, doc_len, hq: int, hkv: int, head_dim: int):
    """Tensors for an ad-hoc small test case with the given document lengths."""
    doc_len = np.asarray(doc_len, dtype=np.int32)
    t = int(doc_len.sum())
    w = Workload(f"small_{seed}", doc_len, t, hq, hkv, head_dim, 1.0 / math.sqrt(head_dim), 1, True, seed)
    return w, w.tensors()
