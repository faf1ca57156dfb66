"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the collectives themselves: it only draws
numbers and describes workload shapes.  Every stream is numpy's counter-based
Philox generator keyed by (seed, rank, tensor id), so any (rank, tensor) can
be regenerated alone and in any order.

The five workloads stand in for what the paper measured and this repository
cannot hold: the OSU micro-benchmark sweeps (Sec. V-B), DS-MoE on the Pile,
DLRM with synthetic batches, and dense Megatron-DeepSpeed (Sec. V-A4).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

BASE_SEED = 230308374


def rng(seed: int, rank: int = 0, tensor: int = 0) -> np.random.Generator:
    """Philox stream for one (seed, rank, tensor) triple."""
    key = (int(seed) & 0xFFFFFFFF) | ((int(rank) & 0xFFFF) << 32) | ((int(tensor) & 0xFFFF) << 48)
    return np.random.Generator(np.random.Philox(key=key))


def f32_bits_to_bf16_trunc(x: np.ndarray) -> np.ndarray:
    """Input preparation only: keep the upper 16 bits of each binary32 value.
    (Truncation, so that no rounding code is shared with either side under
    test; the distribution of the inputs is what matters here.)"""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (a shift, no rounding)."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal(n: int, seed: int, rank: int, tensor: int = 0, std: float = 1.0, bf16: bool = False) -> np.ndarray:
    x = rng(seed, rank, tensor).standard_normal(n, dtype=np.float32)
    if std != 1.0:
        x = x * np.float32(std)
    return f32_bits_to_bf16_trunc(x) if bf16 else x


def uniform_pm1(n: int, seed: int, rank: int, tensor: int = 0, bf16: bool = False) -> np.ndarray:
    """uniform on [-1, 1)."""
    x = rng(seed, rank, tensor).random(n, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
    return f32_bits_to_bf16_trunc(x) if bf16 else x


def uniform01(n: int, seed: int, rank: int, tensor: int = 0) -> np.ndarray:
    return rng(seed, rank, tensor).random(n, dtype=np.float32)


def rank_buffers(P: int, n: int, seed: int, dist: str = "normal", bf16: bool = False, std: float = 1.0) -> List[np.ndarray]:
    if dist == "normal":
        return [normal(n, seed, p, 0, std, bf16) for p in range(P)]
    if dist == "uniform":
        return [uniform_pm1(n, seed, p, 0, bf16) for p in range(P)]
    raise ValueError(dist)


# ---- workload 1: small allreduce --------------------------------------------
@dataclass(frozen=True)
class AllreduceSmall:
    P: int = 4
    n: int = 1 << 20
    seed: int = BASE_SEED + 1

    def buffers(self) -> List[np.ndarray]:
        return rank_buffers(self.P, self.n, self.seed, "normal")


# ---- workload 2: op sweep -----------------------------------------------------
SWEEP_P = 8
SWEEP_BYTES = [1 << k for k in range(12, 29)]       # 4 KiB ... 256 MiB per rank
SWEEP_OPS = ("allreduce", "reduce_scatter", "allgather", "alltoall")
SWEEP_DTYPES = ("f32", "bf16")
SWEEP_SEED = BASE_SEED + 2


# ---- workload 3: MoE dispatch / combine ----------------------------------------
def zipf_ids(T: int, E: int, s: float, seed: int, rank: int, permute: bool = False) -> np.ndarray:
    """Top-1 expert ids with P(expert k-1) proportional to k^-s, k = 1..E (the hottest expert is
    id 0, so hot experts sit together on the low ranks); ``permute`` relabels the experts with a
    seeded permutation instead."""
    w = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w / w.sum())
    u = rng(seed, rank, 1).random(T)
    ids = np.minimum(np.searchsorted(cdf, u, side="right"), E - 1).astype(np.int32)
    if permute:
        perm = rng(seed, 0xFFFF, 2).permutation(E).astype(np.int32)
        ids = perm[ids]
    return ids


@dataclass(frozen=True)
class MoEWorkload:
    P: int = 16
    T: int = 16384
    H: int = 2048
    E: int = 64
    zipf_s: float = 1.2
    capacity_factor: float = 1.25
    seed: int = BASE_SEED + 3

    @property
    def C(self) -> int:
        """Per source rank, per expert capacity."""
        return int(math.ceil(self.capacity_factor * self.T / self.E))

    @property
    def recv_rows(self) -> int:
        """Worst-case rows one rank can receive."""
        return self.P * min(self.T, (self.E // self.P) * self.C)

    def ids(self, rank: int, permute: bool = False) -> np.ndarray:
        return zipf_ids(self.T, self.E, self.zipf_s, self.seed, rank, permute)

    def tokens(self, rank: int) -> np.ndarray:
        return normal(self.T * self.H, self.seed, rank, 3, bf16=True)

    def gate(self, rank: int) -> np.ndarray:
        return uniform01(self.T, self.seed, rank, 4)


# ---- workload 4: DLRM embedding shuffle ----------------------------------------
@dataclass(frozen=True)
class DLRMWorkload:
    P: int = 8
    n_tables: int = 26
    dim: int = 128
    batch: int = 16384
    seed: int = BASE_SEED + 4

    def tables_on(self, rank: int) -> List[int]:
        return list(range(rank, self.n_tables, self.P))

    def pooled(self, rank: int) -> np.ndarray:
        """[T_p, batch, dim] fp32, table-major, flattened."""
        return normal(len(self.tables_on(rank)) * self.batch * self.dim, self.seed, rank, 5)

    def splits(self) -> np.ndarray:
        """S[p, r] = rows rank p sends to rank r in the forward shuffle."""
        bl = self.batch // self.P
        S = np.zeros((self.P, self.P), dtype=np.int64)
        for p in range(self.P):
            S[p, :] = len(self.tables_on(p)) * bl
        return S


# ---- workload 5: dense gradient buckets ----------------------------------------
def gpt_param_shapes(layers: int = 24, hidden: int = 2048, ffn: int = 8192, vocab: int = 50304,
                     seq: int = 2048) -> List[Tuple[str, Tuple[int, ...]]]:
    """GPT-style parameter list in forward order (tied output embedding)."""
    out: List[Tuple[str, Tuple[int, ...]]] = [("wte", (vocab, hidden)), ("wpe", (seq, hidden))]
    for l in range(layers):
        out += [
            (f"h{l}.ln1.w", (hidden,)), (f"h{l}.ln1.b", (hidden,)),
            (f"h{l}.qkv.w", (3 * hidden, hidden)), (f"h{l}.qkv.b", (3 * hidden,)),
            (f"h{l}.proj.w", (hidden, hidden)), (f"h{l}.proj.b", (hidden,)),
            (f"h{l}.ln2.w", (hidden,)), (f"h{l}.ln2.b", (hidden,)),
            (f"h{l}.fc1.w", (ffn, hidden)), (f"h{l}.fc1.b", (ffn,)),
            (f"h{l}.fc2.w", (hidden, ffn)), (f"h{l}.fc2.b", (hidden,)),
        ]
    out += [("lnf.w", (hidden,)), ("lnf.b", (hidden,))]
    return out


@dataclass(frozen=True)
class GradBucketWorkload:
    P: int = 8
    bucket_elems: int = 25_000_000
    std: float = 1e-3
    seed: int = BASE_SEED + 5
    layers: int = 24
    hidden: int = 2048
    ffn: int = 8192
    vocab: int = 50304

    def numel(self) -> List[int]:
        """Element counts in gradient-ready order (reverse of forward)."""
        shapes = gpt_param_shapes(self.layers, self.hidden, self.ffn, self.vocab)
        return [int(np.prod(s)) for _, s in reversed(shapes)]

    def grad(self, rank: int, tensor: int, n: int) -> np.ndarray:
        return normal(n, self.seed, rank, tensor, self.std, bf16=True)
