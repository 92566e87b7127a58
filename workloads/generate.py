"""Value recipes for the synthetic workloads.

Everything is drawn with a `torch.Generator` seeded per problem, on the device the
caller names, so a single problem can be redrawn without the others.  The CPU and
the GPU generators are different streams: parity tests draw once and hand the very
same tensors (copied to the host) to the oracle.

Recipes (all start from Q, K, V ~ N(0,1) i.i.d. per element):
  planted_mean      K rows at `planted_count` random positions are set to
                    3 x (mean of the problem's prompt query rows).
  rope_planted      K is rotated per channel pair (2u, 2u+1) by the angle
                    t * theta_h**(-2u/d) at position t with a per-head base
                    theta_h = 10000 * (1 + h/32); afterwards a fraction of the rows
                    is replaced by keys aligned with the prompt (see `planted`).
  outlier_channels  4 random channels of K are scaled by exp(z), z ~ N(0,1),
                    one z per (problem, channel): a log-normal channel scale.
  planted           a fraction of the K rows, at positions scattered uniformly
                    without replacement, is set to 2*sqrt(d) * qbar/|qbar| where
                    qbar is the mean prompt query row.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np
import torch

from .configs import Request, Workload, problem_seed


def _gen(w: Workload, b: int, l: int, g: int, device) -> torch.Generator:
    gen = torch.Generator(device=device)
    gen.manual_seed(problem_seed(w, b, l, g))
    return gen


def _store(x: torch.Tensor, w: Workload) -> torch.Tensor:
    return x.to(torch.float32 if w.dtype == "f32" else torch.bfloat16).contiguous()


def planted_positions(w: Workload, req: Request, gen: torch.Generator, device) -> torch.Tensor:
    n = w.n_planted(req)
    if n == 0:
        return torch.empty(0, dtype=torch.long, device=device)
    return torch.randperm(req.n_cont, generator=gen, device=device)[:n].sort().values


def make_problem(w: Workload, b: int, l: int, g: int, device="cpu",
                 n_cont: Optional[int] = None) -> Dict[str, torch.Tensor]:
    """Draw one problem: Q [R][d], K [n_cont][d], V [n_cont][d] in storage dtype.

    `n_cont` may shorten the document (used by small test cases that keep a
    workload's value recipe but not its length); planted positions then fall in the
    shortened range.
    """
    req = w.requests[b]
    if n_cont is not None:
        req = Request(n_cont, req.n_que, req.budget)
    d = w.head_dim
    R = w.rows(req)
    gen = _gen(w, b, l, g, device)
    q = torch.randn(R, d, generator=gen, device=device, dtype=torch.float32)
    k = torch.randn(req.n_cont, d, generator=gen, device=device, dtype=torch.float32)
    v = torch.randn(req.n_cont, d, generator=gen, device=device, dtype=torch.float32)
    pos = planted_positions(w, req, gen, device)
    qbar = q.mean(dim=0)

    if w.recipe == "planted_mean":
        k[pos] = 3.0 * qbar
    elif w.recipe == "rope_planted":
        theta = 10000.0 * (1.0 + g / 32.0)
        u = torch.arange(d // 2, device=device, dtype=torch.float64)
        inv = theta ** (-2.0 * u / d)
        t = torch.arange(req.n_cont, device=device, dtype=torch.float64)
        ang = t[:, None] * inv[None, :]
        cs, sn = torch.cos(ang).float(), torch.sin(ang).float()
        ke, ko = k[:, 0::2].clone(), k[:, 1::2].clone()
        k[:, 0::2] = ke * cs - ko * sn
        k[:, 1::2] = ke * sn + ko * cs
        k[pos] = 2.0 * math.sqrt(d) * qbar / qbar.norm()
    elif w.recipe == "outlier_channels":
        ch = torch.randperm(d, generator=gen, device=device)[:4]
        z = torch.randn(4, generator=gen, device=device, dtype=torch.float32)
        k[:, ch] = k[:, ch] * torch.exp(z)[None, :]
    elif w.recipe == "planted":
        k[pos] = 2.0 * math.sqrt(d) * qbar / qbar.norm()
    else:
        raise ValueError(f"unknown recipe {w.recipe!r}")
    return {"Q": _store(q, w), "K": _store(k, w), "V": _store(v, w), "planted": pos}


def make_layer(w: Workload, b: int, l: int, device="cpu", n_cont: Optional[int] = None):
    """All KV heads of one (request, layer): a list of `make_problem` dicts."""
    return [make_problem(w, b, l, g, device, n_cont) for g in range(w.kv_heads)]


def to_numpy_storage(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> host numpy array holding the same bytes.

    float32 stays float32; bfloat16 becomes uint16 bit patterns.
    """
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


def from_numpy_storage(a: np.ndarray, device="cpu") -> torch.Tensor:
    """Inverse of `to_numpy_storage`."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)
