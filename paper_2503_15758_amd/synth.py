"""Seeded synthetic inputs shaped like the paper's GPT-3-like long-context tiles.

This module draws random numbers and nothing else: it holds none of the
method's arithmetic, so both the GPU tests and the CPU oracle's tests may use
it.  Values are drawn in fp32 from N(0, sigma^2) with torch's CPU generator
(bit-identical on every host), then rounded once to the storage dtype; the
oracle is handed those rounded values widened to fp64.

The five workloads follow Table 3 of the paper (heads M and head size H of the
GPT-3-like models) and its sequence lengths (Sec. 4.1: N = 2^13 .. 2^17), cut
into the sqrt(P) x sqrt(P) grid of Sec. 3.2; one tile is N/sqrt(P) rows.
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # "f32" | "bf16"
    heads: int          # B * M
    hdim: int           # H
    seq: int            # N
    grid: int           # sqrt(P)
    causal: bool
    backward: bool
    sigma_qk: float
    seed: int

    @property
    def tile(self):
        return self.seq // self.grid


WORKLOADS = {
    "c1": Workload("c1", "f32", 2, 64, 256, 2, False, False, 1.0, 1001),
    "c2": Workload("c2", "bf16", 16, 128, 8192, 4, False, True, 1.0, 1002),
    "c3": Workload("c3", "bf16", 96, 128, 32768, 8, True, True, 1.0, 1003),
    "c4": Workload("c4", "bf16", 32, 128, 131072, 8, False, True, 1.0, 1004),
    "c5": Workload("c5", "bf16", 8, 128, 262144, 16, False, False, 4.0, 1005),
}


def torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def normal(shape, seed, stream, sigma=1.0, dtype="f32"):
    """N(0, sigma^2) tensor on the CPU; `stream` separates tensors of one seed."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed) * 1000003 + int(stream))
    x = torch.randn(tuple(shape), generator=g, dtype=torch.float32)
    if sigma != 1.0:
        x = x * float(sigma)
    return x.to(torch_dtype(dtype))


# stream ids: one per tensor kind, plus the block index so every block of the
# sequence is an independent draw
Q_STREAM, K_STREAM, V_STREAM, DO_STREAM = 0, 100, 200, 300


def q_block(w, r, rows=None):
    return normal((w.heads, rows or w.tile, w.hdim), w.seed, Q_STREAM + r, w.sigma_qk, w.dtype)


def k_block(w, c, rows=None):
    return normal((w.heads, rows or w.tile, w.hdim), w.seed, K_STREAM + c, w.sigma_qk, w.dtype)


def v_block(w, c, rows=None):
    return normal((w.heads, rows or w.tile, w.hdim), w.seed, V_STREAM + c, 1.0, w.dtype)


def do_block(w, r, rows=None):
    return normal((w.heads, rows or w.tile, w.hdim), w.seed, DO_STREAM + r, 1.0, w.dtype)
