"""Host side of the chunk loop (Method: Document Segmentation).

`ChunkLoop` lays out, once, everything the sequence of prefill steps needs - the
ping-pong cache buffers, the per-step descriptor arrays on host and device, the
r schedule from `finch_schedule` - so that running the loop is nothing but one
`finch_loop` call (or one `finch_step` call per chunk) on a stream, with no
allocation, no host synchronisation and no device-to-host readback in between.

All arithmetic of the method happens inside the library; this file only computes
addresses.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import Batch, Finch, LoopBatch, finch_schedule


class ChunkLoop:
    """Chunked compression of a batch of independent problems.

    problems: sequence of dicts with
        Q       [R][d] tensor, or a list with one [R][d] tensor per step
        K, V    [n_cont][d] document keys / values (device tensors)
        n_que   prompt rows per query head (R = group * n_que)
        budget  k, rows to keep at the end
        Q_doc   optional: [G][chunk][d] queries of a chunk's own tokens (or a list, one
                per step): scoring then also takes those rows, under the causal mask
        K_que   optional: [n_que][d] the prompt's own keys (or a list, one per step):
                the softmax denominators then include them (finch_prompt_lse runs
                at the start of `run`)
    chunk: m, document rows per step.
    history: keep the scores and indices of every step (tests); otherwise one
        scores/idx buffer is reused by all steps.
    constant_budget: keep the whole budget from the first step on instead of growing
        r in proportion to the tokens seen.
    """

    def __init__(self, fin: Finch, problems: Sequence[Dict], chunk: int, history: bool = False,
                 want_scores: bool = True, constant_budget: bool = False):
        self.fin = fin
        self.problems = list(problems)
        self.chunk = int(chunk)
        self.history = history
        dev = fin.device
        P = len(self.problems)
        self.rs: List[List[int]] = []
        self.n_cont: List[int] = []
        for pb in self.problems:
            n = int(pb["K"].shape[0])
            self.n_cont.append(n)
            self.rs.append(finch_schedule(n, self.chunk, int(pb["budget"]), constant_budget))
        self.n_steps = max((len(r) for r in self.rs), default=0)
        d = int(self.problems[0]["K"].shape[1]) if P else 0
        dtype = self.problems[0]["K"].dtype if P else torch.float32
        caps = [max(1, max(r, default=0)) for r in self.rs]
        self.cap_off = [0]
        for c in caps:
            self.cap_off.append(self.cap_off[-1] + c)
        tot_cap = self.cap_off[-1]
        # ping-pong caches, one slab per problem inside each big tensor
        self.kbuf = [torch.zeros(max(1, tot_cap), d, dtype=dtype, device=dev) for _ in range(2)]
        self.vbuf = [torch.zeros(max(1, tot_cap), d, dtype=dtype, device=dev) for _ in range(2)]
        # candidates per (problem, step) and the scores / idx slabs
        nmax = []
        for p in range(P):
            c, best = 0, 1
            for i, r in enumerate(self.rs[p]):
                mi = min(self.chunk, self.n_cont[p] - i * self.chunk)
                best = max(best, c + mi)
                c = r
            nmax.append(best)
        self.n_off = [0]
        for n in nmax:
            self.n_off.append(self.n_off[-1] + n)
        n_hist = self.n_steps if history else 1
        self.want_scores = want_scores or history
        self.scores = (torch.zeros(n_hist, max(1, self.n_off[-1]), dtype=torch.float32, device=dev)
                       if self.want_scores else None)
        self.idx = torch.zeros(n_hist, max(1, tot_cap), dtype=torch.int32, device=dev)
        # per-row term of the prompt's own keys: one slab per problem, per step if
        # the prompt changes from step to step
        self.exact = any(pb.get("K_que") is not None for pb in self.problems)
        self.per_step_prompt = any(isinstance(pb["Q"], (list, tuple)) for pb in self.problems)
        self.row_off = [0]
        for pb in self.problems:
            q0 = pb["Q"][0] if isinstance(pb["Q"], (list, tuple)) else pb["Q"]
            self.row_off.append(self.row_off[-1] + int(q0.shape[0]))
        self.lse_extra = (torch.zeros(self.n_steps if self.per_step_prompt else 1, max(1, self.row_off[-1]),
                                      dtype=torch.float32, device=dev) if self.exact else None)
        self._keep: List[torch.Tensor] = []      # tensors the descriptors point into
        self.batches: List[Batch] = []
        self.active: List[List[int]] = []
        self.step_shapes: List[List[tuple]] = []
        # problems with more steps first, so that the problems present at a step are
        # always the leading slots (what finch_loop asks for)
        order = sorted(range(P), key=lambda p: -len(self.rs[p]))
        all_descs = []
        for i in range(self.n_steps):
            descs, act, shapes = [], [], []
            h = i if history else 0
            for p in order:
                pb = self.problems[p]
                if i >= len(self.rs[p]):
                    continue
                c = self.rs[p][i - 1] if i > 0 else 0
                lo = i * self.chunk
                hi = min(lo + self.chunk, self.n_cont[p])
                r = self.rs[p][i]
                src, dst = i % 2, (i + 1) % 2
                o = self.cap_off[p]
                q = pb["Q"][i] if isinstance(pb["Q"], (list, tuple)) else pb["Q"]
                kq = pb.get("K_que")
                kq = kq[i] if isinstance(kq, (list, tuple)) else kq
                qd = pb.get("Q_doc")
                qd = qd[i] if isinstance(qd, (list, tuple)) else qd
                if qd is not None:
                    # [G][chunk][d] -> the [G * m][d] block of this step (a copy if the chunk is short)
                    qd = qd[:, :hi - lo].reshape(-1, qd.shape[-1])
                    if not qd.is_contiguous():
                        qd = qd.contiguous()
                    self._keep.append(qd)
                extra = None
                if kq is not None:
                    extra = self.lse_extra[i if self.per_step_prompt else 0,
                                           self.row_off[p]:self.row_off[p + 1]]
                descs.append(dict(
                    q=q, k_que=kq, lse_extra=extra, q_doc=qd,
                    k_cache=self.kbuf[src][o:o + c], v_cache=self.vbuf[src][o:o + c],
                    k_chunk=pb["K"][lo:hi], v_chunk=pb["V"][lo:hi],
                    k_out=self.kbuf[dst][o:o + max(r, 1)], v_out=self.vbuf[dst][o:o + max(r, 1)],
                    scores=(self.scores[h, self.n_off[p]:self.n_off[p] + c + (hi - lo)]
                            if self.want_scores else None),
                    idx=self.idx[h, o:o + max(r, 1)],
                    n_que=int(pb["n_que"]), c=c, m=hi - lo, r=r))
                act.append(p)
                shapes.append((c, hi - lo, r))
            self.batches.append(Batch(descs, device=dev))
            self.active.append(act)
            self.step_shapes.append(shapes)
            all_descs.append(descs)
        for b in self.batches:
            fin.reserve(b)
        self.loop_batch = LoopBatch(all_descs, device=dev)
        fin.reserve_loop(self.loop_batch)

    def run(self, stream: Optional[int] = None, per_step: bool = False) -> None:
        """Enqueue the whole loop - one finch_loop call, or with `per_step` one
        finch_step call per chunk; returns without synchronising."""
        if self.exact:
            # every problem is present at step 0; later steps only need it if their prompt differs
            for b in (self.batches if self.per_step_prompt else self.batches[:1]):
                self.fin.prompt_lse(b, stream)
        if per_step:
            for b in self.batches:
                self.fin.step(b, stream)
        else:
            self.fin.loop(self.loop_batch, stream)

    def final_cache(self, p: int):
        """(K~, V~) views of problem p after the last of its steps."""
        steps = len(self.rs[p])
        k = self.rs[p][-1] if steps else 0
        o = self.cap_off[p]
        side = steps % 2
        return self.kbuf[side][o:o + k], self.vbuf[side][o:o + k]

    def step_outputs(self, i: int, p: int):
        """(scores, idx) views written by step i for problem p (history mode)."""
        if not self.history:
            raise RuntimeError("step_outputs needs history=True")
        pos = self.active[i].index(p)
        c, m, r = self.step_shapes[i][pos]
        n, o = self.n_off[p], self.cap_off[p]
        return self.scores[i, n:n + c + m], self.idx[i, o:o + min(r, c + m)]
