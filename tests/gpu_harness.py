"""Shared helpers of the GPU parity tests: compare what the HIP library wrote with
what the CPU oracle computes from the very same input bytes.

Tolerance rule (per step and problem):
  * scores: |gpu - oracle| <= tol * max(|oracle|, 1e-30), tol = 2e-3 for bf16 inputs
    and 1e-5 for fp32 inputs;
  * indices: exactly min(r, N) of them, strictly ascending, in range; where the set
    differs from the oracle's, every differing key must have an oracle score within
    1e-4 relative of the oracle's r-th largest score (a near-tie: either choice is
    right);
  * compacted K/V: bitwise equal to the source rows named by the GPU's own indices.
Because an accepted near-tie swap changes the next step's candidates, a chunk loop
is validated free-running: at each step the oracle is re-run on the cache the GPU
actually holds (rebuilt on the host from the GPU's index history).
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from paper_2408_00167_amd.driver import ChunkLoop

SCORE_TOL = {"bf16": 2e-3, "f32": 1e-5}
SWAP_TOL = 1e-4


def dtype_name(t: torch.Tensor) -> str:
    return "bf16" if t.dtype == torch.bfloat16 else "f32"


def finch_dtype(t: torch.Tensor) -> int:
    return F.FINCH_BF16 if t.dtype == torch.bfloat16 else F.FINCH_F32


def check_scores(gpu_scores: np.ndarray, want: np.ndarray, tol: float, what: str) -> float:
    assert gpu_scores.shape == want.shape, what
    assert np.isfinite(gpu_scores).all(), f"{what}: non-finite scores"
    rel = np.abs(gpu_scores.astype(np.float64) - want) / np.maximum(np.abs(want), 1e-30)
    worst = float(rel.max()) if rel.size else 0.0
    assert worst <= tol, f"{what}: score rel err {worst:.3e} > {tol:g} at key {int(rel.argmax())}"
    return worst


def check_indices(gpu_idx: np.ndarray, want_scores: np.ndarray, r: int, what: str) -> int:
    """Returns the number of accepted near-tie swaps."""
    N = want_scores.shape[0]
    rr = min(r, N)
    assert gpu_idx.shape == (rr,), f"{what}: {gpu_idx.shape} indices, want {rr}"
    if rr == 0:
        return 0
    assert gpu_idx.min() >= 0 and gpu_idx.max() < N, f"{what}: index out of range"
    assert (np.diff(gpu_idx) > 0).all(), f"{what}: indices not strictly ascending"
    want = O.top_r(want_scores, r)
    if np.array_equal(want, gpu_idx):
        return 0
    thr = np.sort(want_scores)[::-1][rr - 1]
    diff = np.setxor1d(want, gpu_idx)
    for j in diff:
        s = want_scores[j]
        rel = abs(s - thr) / max(abs(s), abs(thr), 1e-300)
        assert rel < SWAP_TOL, (f"{what}: key {j} (score {s:.9g}) differs from the oracle's choice "
                                f"but is {rel:.2e} away from the threshold {thr:.9g}")
    return len(diff) // 2


def make_gpu_problem(w: W.Workload, b: int, l: int, g: int, n_cont=None, device="cuda") -> Dict:
    """Draw a workload problem on the GPU and wrap it for ChunkLoop."""
    p = W.make_problem(w, b, l, g, device=device, n_cont=n_cont)
    req = w.requests[b]
    return dict(Q=p["Q"], K=p["K"], V=p["V"], n_que=req.n_que, budget=req.budget,
                planted=p["planted"], id=(b, l, g))


def validate_chunk_loop(loop: ChunkLoop, check: Sequence[int], what: str = "") -> Dict:
    """Free-running validation of the problems in `check` after loop.run()."""
    torch.cuda.synchronize()
    stats = dict(swaps=0, worst_rel=0.0, steps=0)
    for p in check:
        pb = loop.problems[p]
        tol = SCORE_TOL[dtype_name(pb["K"])]
        Kd, Vd = W.to_numpy_storage(pb["K"]), W.to_numpy_storage(pb["V"])
        Kc, Vc = Kd[:0].copy(), Vd[:0].copy()
        pos = np.zeros(0, dtype=np.int64)
        for i, r in enumerate(loop.rs[p]):
            lo, hi = i * loop.chunk, min((i + 1) * loop.chunk, loop.n_cont[p])
            q = pb["Q"][i] if isinstance(pb["Q"], (list, tuple)) else pb["Q"]
            extra = None
            if pb.get("K_que") is not None:
                # checked against the oracle here, then used as the GPU holds it (fp32)
                kq = pb["K_que"][i] if isinstance(pb["K_que"], (list, tuple)) else pb["K_que"]
                extra = loop.lse_extra[i if loop.per_step_prompt else 0,
                                       loop.row_off[p]:loop.row_off[p + 1]].double().cpu().numpy()
                ref = O.prompt_lse(W.to_numpy_storage(q), W.to_numpy_storage(kq), q.shape[0] // pb["n_que"])
                assert np.abs(extra - ref).max() < 1e-5 * max(1.0, np.abs(ref).max()), f"{what}: lse_extra"
            qd = pb.get("Q_doc")
            qd = qd[i] if isinstance(qd, (list, tuple)) else qd
            if qd is not None:
                G = qd.shape[0]
                qd_step = W.to_numpy_storage(qd[:, :hi - lo].reshape(-1, qd.shape[-1]).contiguous())
                want_scores = O.key_scores_conditioned(W.to_numpy_storage(q), qd_step, Kc, Kd[lo:hi], G,
                                                       lse_extra=extra)
            else:
                want_scores = O.key_scores(W.to_numpy_storage(q), Kc, Kd[lo:hi], lse_extra=extra)
            g_scores, g_idx = loop.step_outputs(i, p)
            g_scores, g_idx = g_scores.cpu().numpy(), g_idx.cpu().numpy()
            tag = f"{what} problem {pb.get('id', p)} step {i}"
            stats["worst_rel"] = max(stats["worst_rel"], check_scores(g_scores, want_scores, tol, tag))
            stats["swaps"] += check_indices(g_idx, want_scores, r, tag)
            # the cache the GPU must now hold, from its own choice
            Kc, Vc = O.gather_rows(g_idx, Kc, Kd[lo:hi]), O.gather_rows(g_idx, Vc, Vd[lo:hi])
            pos = np.concatenate([pos, np.arange(lo, hi)])[g_idx]
            stats["steps"] += 1
        Kg, Vg = loop.final_cache(p)
        assert W.to_numpy_storage(Kg).tobytes() == Kc.tobytes(), f"{what} problem {p}: final K differs"
        assert W.to_numpy_storage(Vg).tobytes() == Vc.tobytes(), f"{what} problem {p}: final V differs"
        assert (np.diff(pos) > 0).all(), f"{what} problem {p}: kept positions not ascending"
        assert Kd[pos].tobytes() == Kc.tobytes()
    return stats


def rand_storage(shape, dtype: torch.dtype, gen: torch.Generator, scale=1.0) -> torch.Tensor:
    return (torch.randn(*shape, generator=gen, device="cuda", dtype=torch.float32) * scale).to(dtype)


def single_step_case(fin: F.Finch, specs: Sequence[Dict], dtype: torch.dtype, d: int, group: int,
                     seed: int, null_scores: bool = False):
    """Build one batch of independent single-step problems with random data.

    specs: dicts with n_que, c, m, r.  Returns (batch, tensors per problem).
    """
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    ts: List[Dict] = []
    for sp in specs:
        R, c, m, r = group * sp["n_que"], sp["c"], sp["m"], sp["r"]
        N = c + m
        rr = min(r, N)
        t = dict(
            q=rand_storage((R, d), dtype, gen, sp.get("qscale", 1.0)),
            k_cache=rand_storage((c, d), dtype, gen), v_cache=rand_storage((c, d), dtype, gen),
            k_chunk=rand_storage((m, d), dtype, gen), v_chunk=rand_storage((m, d), dtype, gen),
            k_out=torch.full((max(rr, 1) + 1, d), 7.0, device="cuda").to(dtype),
            v_out=torch.full((max(rr, 1) + 1, d), 7.0, device="cuda").to(dtype),
            scores=None if null_scores else torch.full((max(N, 1) + 1,), -5.0, device="cuda"),
            idx=torch.full((max(rr, 1) + 1,), -9, dtype=torch.int32, device="cuda"),
            n_que=sp["n_que"], c=c, m=m, r=r)
        t["group"] = group
        if sp.get("doc_rows"):
            # queries of the chunk's own tokens, head by head
            t["q_doc"] = rand_storage((group * m, d), dtype, gen, sp.get("qscale", 1.0)) if m > 0 else None
            if sp.get("no_prompt"):
                t["q"] = None
        if sp.get("prompt_keys"):
            # the prompt's own keys and room for the per-row term they add to the denominator
            t["k_que"] = rand_storage((sp["n_que"], d), dtype, gen, sp.get("qscale", 1.0))
            t["lse_extra"] = torch.full((R + 1,), -77.0, device="cuda")
        if "kramp" in sp and m > 0:
            # key magnitudes change steadily along the chunk (from 1x to kramp x)
            ramp = torch.logspace(0.0, float(np.log10(sp["kramp"])), m, device="cuda").unsqueeze(1)
            t["k_chunk"] = (t["k_chunk"].float() * ramp).to(dtype)
        ts.append(t)
    descs = []
    for t in ts:
        dsc = dict(t)
        N, rr = t["c"] + t["m"], min(t["r"], t["c"] + t["m"])
        # hand the library exactly-sized views; the extra element/row is a guard
        dsc["k_out"], dsc["v_out"] = t["k_out"][:max(rr, 1)], t["v_out"][:max(rr, 1)]
        dsc["idx"] = t["idx"][:max(rr, 1)]
        if t["scores"] is not None:
            dsc["scores"] = t["scores"][:max(N, 1)]
        if t.get("lse_extra") is not None:
            dsc["lse_extra"] = t["lse_extra"][:-1]
        descs.append(dsc)
    return F.Batch(descs), ts


def check_repositioned(t: Dict, Kc, Kk, Vc, Vk, idx, rr, pairing, order, base, tag) -> float:
    """K', V' of one problem against the oracle's re-positioned compaction.  Slots
    by rank are decided from the scores the GPU itself holds (fp32), with the
    oracle's rule; keys within rounding of the fp64 rotation; values bit for bit."""
    Kout, Vout = W.to_numpy_storage(t["k_out"]), W.to_numpy_storage(t["v_out"])
    gscores = t["scores"].cpu().numpy()[:t["c"] + t["m"]] if t["scores"] is not None else None
    Kw, Vw, slots = O.compact_repositioned(idx[:rr], gscores, Kc, Kk, Vc, Vk, base, pairing, order)
    assert Vout[:rr].tobytes() == Vw.tobytes(), f"{tag}: V rows"
    got = O.widen(Kout[:rr])
    rowmax = np.abs(Kw).max(axis=1, keepdims=True) if rr else np.zeros((0, 1))
    rel = 0.004 if dtype_name(t["k_out"]) == "bf16" else 0.0
    err = np.abs(got - Kw)
    bound = rel * np.abs(Kw) + 1e-5 * rowmax
    assert (err <= bound).all(), f"{tag}: re-positioned K off by {float((err - bound).max()):.3e}"
    # a candidate that keeps its position keeps its bits
    both = np.concatenate([Kc, Kk], axis=0)
    for ti in np.nonzero(slots == idx[:rr])[0]:
        assert Kout[slots[ti]].tobytes() == both[idx[ti]].tobytes(), f"{tag}: unmoved key changed"
    return float((err / np.maximum(rowmax, 1e-30)).max()) if rr else 0.0


def validate_single_step(ts: Sequence[Dict], what: str, check_scores_too: bool = True,
                         repos=None) -> Dict:
    """`repos` = (pairing or None, order, base) when re-positioning is switched on."""
    torch.cuda.synchronize()
    stats = dict(swaps=0, worst_rel=0.0, worst_rot=0.0)
    for n, t in enumerate(ts):
        tol = SCORE_TOL[dtype_name(t["k_out"])]
        N, r = t["c"] + t["m"], t["r"]
        rr = min(r, N)
        Kc, Kk = W.to_numpy_storage(t["k_cache"]), W.to_numpy_storage(t["k_chunk"])
        Vc, Vk = W.to_numpy_storage(t["v_cache"]), W.to_numpy_storage(t["v_chunk"])
        extra = None
        if t.get("lse_extra") is not None:
            # the scoring is checked with the term the GPU was given (itself checked apart)
            extra = t["lse_extra"][:-1].double().cpu().numpy()
            assert float(t["lse_extra"][-1]) == -77.0, "wrote past the end of lse_extra"
        if t.get("q_doc") is not None or t["q"] is None:
            want = O.key_scores_conditioned(
                None if t["q"] is None else W.to_numpy_storage(t["q"]),
                None if t.get("q_doc") is None else W.to_numpy_storage(t["q_doc"]), Kc, Kk, t["group"],
                lse_extra=extra)
        else:
            want = O.key_scores(W.to_numpy_storage(t["q"]), Kc, Kk, lse_extra=extra)
        tag = f"{what} problem {n} (n_que={t['n_que']}, c={t['c']}, m={t['m']}, r={r})"
        if check_scores_too and t["scores"] is not None:
            got = t["scores"].cpu().numpy()
            stats["worst_rel"] = max(stats["worst_rel"], check_scores(got[:N], want, tol, tag))
            assert got[N] == -5.0 or N == 0, f"{tag}: wrote past the end of scores"
        idx = t["idx"].cpu().numpy()
        stats["swaps"] += check_indices(idx[:rr], want, r, tag)
        assert idx[max(rr, 1)] == -9, f"{tag}: wrote past the end of idx"
        if rr == 0:
            assert idx[0] == -9
        Kout, Vout = W.to_numpy_storage(t["k_out"]), W.to_numpy_storage(t["v_out"])
        if repos is None:
            assert Kout[:rr].tobytes() == O.gather_rows(idx[:rr], Kc, Kk).tobytes(), f"{tag}: K rows"
            assert Vout[:rr].tobytes() == O.gather_rows(idx[:rr], Vc, Vk).tobytes(), f"{tag}: V rows"
        else:
            stats["worst_rot"] = max(stats["worst_rot"],
                                     check_repositioned(t, Kc, Kk, Vc, Vk, idx, rr, *repos, tag))
        guard = W.to_numpy_storage(torch.full((1, Kout.shape[1]), 7.0).to(t["k_out"].dtype))
        assert Kout[rr:].tobytes() == np.repeat(guard, Kout.shape[0] - rr, axis=0).tobytes(), \
            f"{tag}: rows beyond r were touched"
        assert Vout[rr:].tobytes() == np.repeat(guard, Vout.shape[0] - rr, axis=0).tobytes()
    return stats
