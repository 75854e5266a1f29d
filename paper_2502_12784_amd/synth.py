"""Seeded synthetic attention inputs shared by the tests, the smoke check and bench.py.

This module holds none of the method's arithmetic: it only draws normal random
numbers, rounds them to the 16-bit storage type and widens them back exactly.
The paper's own workload is random numbers in fp16 (Sec. 4.1, "Dataset"), so
synthetic inputs of these shapes are the workload, not a stand-in for one.

Recipe (identical for every caller): ``SeedSequence(seed).spawn(4)`` gives one
child stream each for Q, K, V, dO in that order; each tensor is
``standard_normal(float32) * sigma`` rounded to nearest-even fp16 / bf16.  The
16-bit patterns go to the GPU; the same values widened exactly to float64 go to
the CPU oracle, so a comparison measures kernel error, not input rounding.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

F16 = "f16"
BF16 = "bf16"


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    dtype: str
    causal: bool
    sigma_qk: float
    seed: int
    note: str = ""

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def fwd_flops(self) -> float:
        """Counted forward flops: two N x N x d contractions per head; the causal
        half is counted as half (the paper's Sec. 4.2.1 convention)."""
        f = 4.0 * self.B * self.H * self.N * self.N * self.d
        return f / 2 if self.causal else f

    @property
    def bwd_flops(self) -> float:
        """Five N x N x d contractions (Eq. 4 plus the recomputed S)."""
        return 2.5 * self.fwd_flops


# The five benchmark configurations (C1..C5).  C5 draws Q and K with variance 3
# so that logits scale*q.k have standard deviation 3.
WORKLOADS = {
    "C1": Workload("C1", 1, 2, 128, 64, F16, False, 1.0, 1001, "tiny"),
    "C2": Workload("C2", 8, 12, 512, 64, F16, False, 1.0, 1002, "BERT-base-like"),
    "C3": Workload("C3", 8, 16, 1024, 64, F16, True, 1.0, 1003, "GPT-style causal"),
    "C4": Workload("C4", 4, 16, 4096, 128, BF16, True, 1.0, 1004, "larger-head causal"),
    "C5": Workload("C5", 2, 16, 8192, 64, F16, False, math.sqrt(3.0), 1005, "long sequence, logits std 3"),
}


def round_to_bits(x32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 -> uint16 bit patterns of fp16 / bf16 (round to nearest even)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == F16:
        return x32.astype(np.float16).view(np.uint16)
    if dtype == BF16:
        u = x32.view(np.uint32).astype(np.uint64)
        lsb = (u >> 16) & 1
        r = (u + 0x7FFF + lsb) >> 16
        return r.astype(np.uint16)
    raise ValueError(dtype)


def bits_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    """uint16 bit patterns -> exact float64 values."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == F16:
        return bits.view(np.float16).astype(np.float64)
    if dtype == BF16:
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def make_inputs(B, H, N, d, dtype, seed, sigma_qk=1.0, sigma_v=1.0, sigma_do=1.0, heads=None,
                Nk=None):
    """Return {"Q","K","V","dO"} -> uint16 arrays [B,H,N,d] (bit patterns).

    ``Nk``: number of key/value rows if it differs from the N query rows
    (cross-attention); K and V are then [B,H,Nk,d].

    ``heads``: optional list of flat (b*H+h) indices; if given, only those heads
    are returned (shape [len(heads),1,N,d]) but drawn exactly as in the full
    tensor, so a sampled oracle run sees the same numbers as the full GPU run.
    """
    children = np.random.SeedSequence(seed).spawn(4)
    sig = {"Q": sigma_qk, "K": sigma_qk, "V": sigma_v, "dO": sigma_do}
    out = {}
    for name, child in zip(("Q", "K", "V", "dO"), children):
        rng = np.random.default_rng(child)
        rows = Nk if (Nk is not None and name in ("K", "V")) else N
        x = rng.standard_normal((B * H, rows, d), dtype=np.float32)
        if heads is not None:
            x = x[list(heads)]
            x = x.reshape(len(heads), 1, rows, d)
        else:
            x = x.reshape(B, H, rows, d)
        x = x * np.float32(sig[name])
        out[name] = round_to_bits(x, dtype)
    return out


def make_workload_inputs(w: Workload, heads=None):
    return make_inputs(w.B, w.H, w.N, w.d, w.dtype, w.seed, sigma_qk=w.sigma_qk, heads=heads)
