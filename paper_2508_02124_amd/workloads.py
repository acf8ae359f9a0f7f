"""Seeded synthetic inputs shaped like the paper's kernel benchmark.

This module only draws random numbers and rounds them to the storage dtype; it
contains none of the method's arithmetic and is the one piece of code the test
oracle and the HIP path both consume.

Shapes follow the paper's speed-benchmark table (32 query heads, 8 kv heads,
head dim 128, bf16; Appendix B, "Speed Benchmark Configurations"), the window
of its 1.7B model (2048; Appendix B, scaling-law table) and its 16K
fine-tuning length (Section 5.3).  Values: Q, K, V, dO ~ N(0, 1); mask
projection w_h ~ N(0, 1/d); gate A_h = -U(0.5, 2).  Because V is i.i.d., the
content scores are i.i.d. over keys, so kept keys are scattered uniformly --
the worst case for any skipping of contiguous key blocks.

Layouts: Q, dO [T, H_q, d]; K, V [T, H_kv, d]; W [H_q, d]; A [H_q];
cu_seqlens [n_docs + 1] int32.  bf16 tensors are returned as uint16 bit
patterns (round-to-nearest-even from the fp32 draw) plus helpers to widen them.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    H_q: int
    H_kv: int
    d: int
    k: int
    seqlens: tuple | None = None      # fixed-length documents; None => drawn (varlen)
    total_tokens: int = 0             # varlen only
    len_lo: int = 0
    len_hi: int = 0
    causal: bool = True
    backward: bool = True

    def with_k(self, k):
        return replace(self, k=k, name=f"{self.name}_k{k}")


CONFIGS = {
    # tiny causal case the oracle finishes in seconds (fp32 and bf16)
    "cfg1": Workload("cfg1", 1001, H_q=2, H_kv=2, d=64, k=64, seqlens=(256,)),
    # GQA training shape
    "cfg2": Workload("cfg2", 1002, H_q=16, H_kv=4, d=128, k=1024, seqlens=(4096, 4096)),
    # headline: long context
    "cfg3": Workload("cfg3", 1003, H_q=32, H_kv=8, d=128, k=2048, seqlens=(16384,)),
    # very long, forward only, k swept by the caller via with_k()
    "cfg4": Workload("cfg4", 1004, H_q=32, H_kv=8, d=128, k=4096, seqlens=(65536,), backward=False),
    # varlen packed batch
    "cfg5": Workload("cfg5", 1005, H_q=16, H_kv=16, d=64, k=512, total_tokens=65536,
                     len_lo=512, len_hi=8192),
    # not one of the benchmark's shapes: the headline length at head dimension 256 with half the
    # heads (the same algorithmic FLOPs as cfg3), for the wider-head variant of the kernels
    "cfg3_d256": Workload("cfg3_d256", 1006, H_q=16, H_kv=4, d=256, k=2048, seqlens=(16384,)),
}


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Inputs:
    wl: Workload
    cu_seqlens: np.ndarray            # int32 [n_docs + 1]
    Q: np.ndarray                     # float32 values (already rounded to the storage dtype)
    K: np.ndarray
    V: np.ndarray
    dO: np.ndarray
    W: np.ndarray                     # float32 [H_q, d]
    A: np.ndarray                     # float32 [H_q]
    dtype: str = "bf16"
    bits: dict = field(default_factory=dict)   # name -> uint16 bit patterns (bf16 only)

    @property
    def T(self):
        return int(self.cu_seqlens[-1])

    @property
    def max_seqlen(self):
        return int(np.diff(self.cu_seqlens).max())


def draw_seqlens(rng, total, lo, hi):
    """Lengths uniform in [lo, hi], drawn until the running total reaches
    `total`; the last document is truncated to fit (it may be shorter than lo)."""
    lens, run = [], 0
    while run < total:
        n = int(rng.integers(lo, hi + 1))
        n = min(n, total - run)
        lens.append(n)
        run += n
    return tuple(lens)


def make_inputs(wl: Workload, dtype="bf16"):
    """Draw order is fixed: Q, K, V, dO, W, A, then (varlen) the lengths."""
    rng = np.random.default_rng(wl.seed)
    T = sum(wl.seqlens) if wl.seqlens is not None else wl.total_tokens

    def normal(shape):
        return rng.standard_normal(shape, dtype=np.float32)

    Q = normal((T, wl.H_q, wl.d))
    K = normal((T, wl.H_kv, wl.d))
    V = normal((T, wl.H_kv, wl.d))
    dO = normal((T, wl.H_q, wl.d))
    W = (normal((wl.H_q, wl.d)) / np.float32(np.sqrt(wl.d))).astype(np.float32)
    A = (-rng.uniform(0.5, 2.0, size=wl.H_q)).astype(np.float32)
    seqlens = wl.seqlens if wl.seqlens is not None else draw_seqlens(rng, T, wl.len_lo, wl.len_hi)
    cu = np.concatenate([[0], np.cumsum(seqlens)]).astype(np.int32)
    inp = Inputs(wl, cu, Q, K, V, dO, W, A, dtype=dtype)
    if dtype == "bf16":
        for name in ("Q", "K", "V", "dO"):
            b = f32_to_bf16_bits(getattr(inp, name))
            inp.bits[name] = b
            setattr(inp, name, bf16_bits_to_f32(b))
    elif dtype != "f32":
        raise ValueError(dtype)
    return inp


def small_workload(name, seed, H_q, H_kv, d, k, seqlens, causal=True):
    """Ad-hoc workload for parity tests (same value distributions)."""
    return Workload(name, seed, H_q=H_q, H_kv=H_kv, d=d, k=k, seqlens=tuple(seqlens), causal=causal)
