"""Seeded synthetic inputs for the fused tensor-parallel GEMM workloads.

This module only draws random tensors and names the workload shapes.  It contains none of the
method's arithmetic and is the one module that both the GPU tests/benchmark and the CPU oracle's
callers use, so that both sides see bit-identical inputs.

Shapes follow the paper's op-level evaluation (Sec. 5.1): GEMMs of one tensor-parallel rank of
a transformer layer, 8-way tensor parallelism, bf16, activations ~ N(0,1) and weights
~ N(0, 0.02) (0.02 is the standard deviation).  All tensors are drawn in fp32 on the CPU from
`torch.Generator().manual_seed(seed)` and rounded once to bf16; the rounded values are the
inputs of every implementation.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch

BASE_SEED = 20240606


@dataclass(frozen=True)
class Workload:
    name: str
    op: str                 # "rs" (GEMM-ReduceScatter) or "ag" (AllGather-GEMM)
    M: int                  # rows of the local GEMM (all tokens)
    N: int
    K: int
    R: int                  # tensor-parallel degree (virtual ranks)
    partial_dtype: str = "bf16"   # rs only
    out_dtype: str = "bf16"
    a_dist: tuple = ("normal", 1.0)
    b_dist: tuple = ("normal", 0.02)
    peer_dist: tuple = ("normal", 1.0)
    seed: int = BASE_SEED
    tile: tuple | None = None     # forced (BM, BN) if the workload fixes one

    @property
    def S(self) -> int:
        return self.M // self.R

    @property
    def flops(self) -> float:
        return 2.0 * self.M * self.N * self.K


def _decode(M: int, op: str) -> Workload:
    if op == "ag":
        return Workload(f"c5_ag_m{M}", "ag", M, 3584, 8192, 8, seed=BASE_SEED + 4)
    return Workload(f"c5_rs_m{M}", "rs", M, 8192, 3584, 8, seed=BASE_SEED + 4)


WORKLOADS = {
    # small correctness case: fp32 partial and fp32 output, 64x64 tiles
    "c1_rs": Workload("c1_rs", "rs", 128, 256, 256, 2, partial_dtype="f32", out_dtype="f32",
                      a_dist=("uniform", 1.0), b_dist=("uniform", 1.0), seed=BASE_SEED + 0,
                      tile=(64, 64)),
    # Llama-2-70B-like MLP at TP=8, 4096 tokens
    "c2_ag": Workload("c2_ag", "ag", 4096, 3584, 8192, 8, seed=BASE_SEED + 1),
    "c3_rs": Workload("c3_rs", "rs", 4096, 8192, 3584, 8, seed=BASE_SEED + 2),
    # GPT-3-175B-like layer at TP=8, 8192 tokens
    "c4_ag": Workload("c4_ag", "ag", 8192, 4608, 12288, 8, seed=BASE_SEED + 3),
    "c4_rs": Workload("c4_rs", "rs", 8192, 12288, 1536, 8, seed=BASE_SEED + 3),
    # decode
    **{w.name: w for w in (_decode(m, op) for m in (8, 64, 256) for op in ("ag", "rs"))},
    # the op-level sweep of the paper's evaluation (Sec. 5.1): GPT-3-175B MLP at TP=8, local (n, k) =
    # (6144, 12288) for AllGather-GEMM and (12288, 6144) for GEMM-ReduceScatter, m tokens (m = 8 and 64:
    # the same weight shards at decode batch sizes)
    **{f"op_ag_m{m}": Workload(f"op_ag_m{m}", "ag", m, 6144, 12288, 8, seed=BASE_SEED + 5) for m in (8, 64, 512, 2048, 8192)},
    **{f"op_rs_m{m}": Workload(f"op_rs_m{m}", "rs", m, 12288, 6144, 8, seed=BASE_SEED + 6) for m in (8, 64, 512, 2048, 8192)},
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some dimensions replaced (reduced-size parity cases)."""
    return replace(w, **kw)


def _draw(gen: torch.Generator, shape, dist) -> torch.Tensor:
    kind, scale = dist
    if kind == "normal":
        return torch.randn(shape, generator=gen, dtype=torch.float32) * scale
    if kind == "uniform":
        return (torch.rand(shape, generator=gen, dtype=torch.float32) * 2.0 - 1.0) * scale
    if kind == "int":          # integers in [-scale, scale], exact in bf16 for scale <= 256
        s = int(scale)
        return torch.randint(-s, s + 1, shape, generator=gen).to(torch.float32)
    raise ValueError(kind)


def _as(t: torch.Tensor, dtype: str) -> torch.Tensor:
    return t.to(torch.bfloat16) if dtype == "bf16" else t.to(torch.float32)


def make_rs_inputs(w: Workload, rank: int):
    """A [M,K] bf16, B [K,N] bf16, peers: list of R tensors [M,N] (entry `rank` is None)."""
    gen = torch.Generator().manual_seed(w.seed * 16 + rank)
    A = _as(_draw(gen, (w.M, w.K), w.a_dist), "bf16")
    B = _as(_draw(gen, (w.K, w.N), w.b_dist), "bf16")
    peers = [None if j == rank else _as(_draw(gen, (w.M, w.N), w.peer_dist), w.partial_dtype)
             for j in range(w.R)]
    return A, B, peers


def make_ag_inputs(w: Workload, rank: int):
    """A_chunks: list of R tensors [M/R,K] bf16; B [K,N] bf16; arrival_order: seeded random
    permutation of the remote ranks (the order the copy driver releases chunks in)."""
    gen = torch.Generator().manual_seed(w.seed * 16 + rank)
    chunks = [_as(_draw(gen, (w.S, w.K), w.a_dist), "bf16") for _ in range(w.R)]
    B = _as(_draw(gen, (w.K, w.N), w.b_dist), "bf16")
    remote = [c for c in range(w.R) if c != rank]
    perm = torch.randperm(len(remote), generator=gen).tolist()
    return chunks, B, [remote[p] for p in perm]


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """torch CPU tensor -> numpy in the oracle's conventions (bf16 as uint16 bit patterns)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(t.dtype)
