"""The five synthetic workloads (C1..C5) the selection path is tested and timed on.

Each stands in for prompts and documents of a public long-context benchmark run
through a Llama-2 / Mistral / Llama-3 shaped model: only the head geometry, chunk
sizes, prompt lengths and compression ratios are taken over, every value is drawn
from a seeded generator.  A *problem* is one (request, layer, KV head) triple; its
query block stacks the G = q_heads / kv_heads query heads of the KV group, so it
has R = G * n_que rows.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Iterator, Tuple

import numpy as np


@dataclass(frozen=True)
class Request:
    n_cont: int      # document (context) tokens
    n_que: int       # prompt rows per query head
    budget: int      # k: rows kept per KV head at the end


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" or "bf16": storage type of Q, K, V
    layers: int
    q_heads: int
    kv_heads: int
    head_dim: int
    chunk: int                 # m: document tokens per step
    seed: int
    recipe: str                # which value recipe generate.py applies
    requests: Tuple[Request, ...]
    planted_count: int = 0     # planted keys per problem (absolute) ...
    planted_frac: float = 0.0  # ... or as a fraction of n_cont
    note: str = ""

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads

    def rows(self, req: Request) -> int:
        """R: stacked prompt rows of one KV group."""
        return self.group * req.n_que

    @property
    def n_problems(self) -> int:
        return len(self.requests) * self.layers * self.kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def n_planted(self, req: Request) -> int:
        if self.planted_count:
            return self.planted_count
        return int(round(self.planted_frac * req.n_cont))


def _ragged_requests(seed: int, n: int) -> Tuple[Request, ...]:
    rng = np.random.default_rng(seed)
    lens = rng.integers(2048, 65536, size=n, endpoint=True)
    ques = rng.integers(16, 128, size=n, endpoint=True)
    return tuple(Request(int(L), int(q), int(L) // 32) for L, q in zip(lens, ques))


WORKLOADS = {
    "C1": Workload("C1", "f32", layers=1, q_heads=4, kv_heads=4, head_dim=64, chunk=256,
                   seed=0, recipe="planted_mean", requests=(Request(1024, 16, 64),),
                   planted_count=8,
                   note="tiny fp32; 8 planted keys per head = 3 x mean prompt query"),
    "C2": Workload("C2", "bf16", layers=32, q_heads=32, kv_heads=32, head_dim=128, chunk=512,
                   seed=1, recipe="rope_planted", requests=(Request(4096, 32, 1024),),
                   planted_frac=0.01,
                   note="Llama-2-7B-shaped MHA; RoPE-like rotation; 1% aligned keys"),
    "C3": Workload("C3", "bf16", layers=32, q_heads=32, kv_heads=8, head_dim=128, chunk=2048,
                   seed=2, recipe="outlier_channels", requests=(Request(32768, 64, 2048),),
                   note="Mistral-7B-shaped GQA; log-normal scale on 4 outlier channels"),
    "C4": Workload("C4", "bf16", layers=32, q_heads=32, kv_heads=8, head_dim=128, chunk=4096,
                   seed=3, recipe="planted", requests=(Request(131072, 48, 1408),),
                   planted_frac=0.005,
                   note="Llama-3-8B-shaped GQA, 131072 tokens: the roofline workload"),
    "C5": Workload("C5", "bf16", layers=32, q_heads=32, kv_heads=8, head_dim=128, chunk=2048,
                   seed=4, recipe="planted", requests=_ragged_requests(4, 16),
                   planted_frac=0.005,
                   note="ragged batch of 16 requests, Llama-3-8B-shaped"),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def problems_of(w: Workload) -> Iterator[Tuple[int, int, int]]:
    """All (request, layer, kv_head) triples in the canonical order."""
    for b in range(len(w.requests)):
        for l in range(w.layers):
            for g in range(w.kv_heads):
                yield b, l, g


_MASK = (1 << 64) - 1


def _mix(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK
    return x ^ (x >> 31)


def problem_seed(w: Workload, b: int, l: int, g: int) -> int:
    """A 63-bit seed per problem so any single problem can be redrawn alone."""
    h = _mix(w.seed)
    for v in (b, l, g):
        h = _mix(h ^ _mix(v + 1))
    return h & ((1 << 63) - 1)
