"""The options beyond the default path at the sizes of workload C4 (chunks of 4096
tokens, G = 4, 48 prompt rows per head, caches growing to 1408 rows), through whole
chunk loops, every step of every problem against the oracle: document-row
conditioning, layer-wise selection, re-positioning, the paper-exact denominator."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from paper_2408_00167_amd.driver import ChunkLoop
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def c4_problems(n, n_cont=None, layer=0):
    w = W.get_workload("C4")
    return w, [H.make_gpu_problem(w, 0, layer + g // 8, g % 8, n_cont=n_cont) for g in range(n)]


@pytest.mark.timeout(900)
def test_c4_document_rows_whole_loop():
    """m = 4096 document rows per head and step (65 row chunks of 256 per head), caches
    of 352 ... 1056 rows: four steps of two problems in one launch."""
    say("C4 document rows")
    w, probs = c4_problems(2, n_cont=4 * 4096)
    gen = torch.Generator(device="cuda"); gen.manual_seed(77)
    for pb in probs:
        pb["budget"] = 1408
        pb["Q_doc"] = H.rand_storage((4 * 4096, 128), torch.bfloat16, gen).reshape(4, 4096, 128)
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    loop = ChunkLoop(fin, probs, 4096, history=True)
    assert loop.rs[0] == [352, 704, 1056, 1408]
    loop.run()
    st = H.validate_chunk_loop(loop, [0, 1], "C4 document rows")
    say(f"  {st}")
    fin.close()


def validate_layer_loop(loop, heads, what):
    """Free-running check of one layer (its KV heads share every selection): per step the
    oracle's per-head scores on the cache the GPU holds, their sum, and the shared indices."""
    torch.cuda.synchronize()
    L = len(heads)
    Kd = [W.to_numpy_storage(loop.problems[p]["K"]) for p in heads]
    Vd = [W.to_numpy_storage(loop.problems[p]["V"]) for p in heads]
    Kc = [k[:0].copy() for k in Kd]
    Vc = [v[:0].copy() for v in Vd]
    swaps, worst = 0, 0.0
    p0 = heads[0]
    for i, r in enumerate(loop.rs[p0]):
        lo, hi = i * loop.chunk, min((i + 1) * loop.chunk, loop.n_cont[p0])
        per_head, fp32_sum = [], None
        for h, p in enumerate(heads):
            want = O.key_scores(W.to_numpy_storage(loop.problems[p]["Q"]), Kc[h], Kd[h][lo:hi])
            g_scores, _ = loop.step_outputs(i, p)
            g = g_scores.cpu().numpy()
            worst = max(worst, H.check_scores(g, want, H.SCORE_TOL["bf16"], f"{what} head {h} step {i}"))
            per_head.append(want)
            fp32_sum = g.copy() if fp32_sum is None else fp32_sum + g
        total = O.layer_scores(per_head)
        g_idx = loop.step_outputs(i, p0)[1].cpu().numpy()
        swaps += H.check_indices(g_idx, total, r, f"{what} step {i}")
        # the decision in the precision the GPU takes it in: fp32 sums, head by head
        assert g_idx.tolist() == O.top_r(fp32_sum, r).tolist(), f"{what} step {i}: not the top r of the fp32 sums"
        for h, p in enumerate(heads):
            assert torch.equal(loop.step_outputs(i, p)[1], loop.step_outputs(i, p0)[1]), f"{what} step {i}: heads disagree"
            Kc[h], Vc[h] = O.gather_rows(g_idx, Kc[h], Kd[h][lo:hi]), O.gather_rows(g_idx, Vc[h], Vd[h][lo:hi])
    for h, p in enumerate(heads):
        Kg, Vg = loop.final_cache(p)
        assert W.to_numpy_storage(Kg).tobytes() == Kc[h].tobytes(), f"{what} head {h}: final K"
        assert W.to_numpy_storage(Vg).tobytes() == Vc[h].tobytes(), f"{what} head {h}: final V"
    return dict(swaps=swaps, worst_rel=worst, steps=len(loop.rs[p0]))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("per_step,path", [(False, "separate"), (True, "separate"), (False, "owner"), (True, "owner")])
def test_c4_layer_wise_selection_whole_loop(per_step, path):
    """Two layers of C4 (8 KV heads each, one selection per step for all of them) through
    all 32 chunk steps: one kernel per stage, or one workgroup per problem (whole loop
    in one launch, or step by step) with the layer's workgroups exchanging their scores."""
    say(f"C4 layer-wise selection, per_step={per_step} {path}")
    w, probs = c4_problems(16)      # two layers' worth of heads: two runs of 8
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_OWNER if path == "owner" else F.FINCH_PATH_SEPARATE)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 8)
    loop = ChunkLoop(fin, probs, w.chunk, history=True)
    assert loop.n_steps == 32
    loop.run(per_step=per_step)
    assert fin.workspace_status() == 0
    for run in range(2):
        st = validate_layer_loop(loop, list(range(8 * run, 8 * run + 8)), f"C4 layer run {run}")
        say(f"  run {run}: {st}")
    fin.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("order", ["ascending", "rank"])
def test_c4_repositioned_whole_loop(order):
    """Keys rotated to their slots (ascending, or by relevance as in the paper's worked
    example) while they are compacted, rotary pairs d/2 apart, all 32 steps: step by step
    with the cache the GPU holds read back after every step and every step against the
    oracle, then the whole loop in one launch, which must give the same bits."""
    say(f"C4 re-positioning, {order} slots")
    base = 500000.0
    w, probs = c4_problems(4)
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_RANK if order == "rank" else F.FINCH_ORDER_ASCENDING, base)
    a = ChunkLoop(fin, probs, w.chunk, history=True)
    check = [0, 3]
    caches = {p: (np.zeros((0, 128), np.uint16), np.zeros((0, 128), np.uint16)) for p in check}
    worst_rot = 0.0
    for i, b in enumerate(a.batches):
        fin.step(b)
        torch.cuda.synchronize()
        lo, hi = i * a.chunk, (i + 1) * a.chunk
        side = (i + 1) % 2
        for p in check:
            pb = a.problems[p]
            Kc, Vc = caches[p]
            Kk, Vk = W.to_numpy_storage(pb["K"][lo:hi]), W.to_numpy_storage(pb["V"][lo:hi])
            want = O.key_scores(W.to_numpy_storage(pb["Q"]), Kc, Kk)
            g_scores, g_idx = a.step_outputs(i, p)
            H.check_scores(g_scores.cpu().numpy(), want, H.SCORE_TOL["bf16"], f"reposition problem {p} step {i}")
            idx = g_idx.cpu().numpy()
            r = a.rs[p][i]
            H.check_indices(idx, want, r, f"reposition problem {p} step {i}")
            o = a.cap_off[p]
            t = dict(k_out=a.kbuf[side][o:o + r], v_out=a.vbuf[side][o:o + r], scores=g_scores, c=Kc.shape[0], m=hi - lo)
            worst_rot = max(worst_rot, H.check_repositioned(t, Kc, Kk, Vc, Vk, idx, r, "half", order, base,
                                                            f"reposition problem {p} step {i}"))
            caches[p] = (W.to_numpy_storage(a.kbuf[side][o:o + r]).copy(), W.to_numpy_storage(a.vbuf[side][o:o + r]).copy())
    say(f"  step by step ok, worst rotation error (relative to the row maximum) {worst_rot:.2e}")
    b = ChunkLoop(fin, probs, w.chunk, history=True)
    b.run()
    torch.cuda.synchronize()
    assert torch.equal(a.scores, b.scores) and torch.equal(a.idx, b.idx)
    for p in range(len(probs)):
        for x, y in zip(a.final_cache(p), b.final_cache(p)):
            assert torch.equal(x, y), f"whole loop differs from step by step, problem {p}"
    fin.close()


@pytest.mark.timeout(900)
def test_c4_exact_denominator_whole_loop():
    """The prompt's own keys in every denominator, all 32 steps of four C4 problems in one
    launch."""
    say("C4 exact denominator")
    w, probs = c4_problems(4)
    gen = torch.Generator(device="cuda"); gen.manual_seed(78)
    for pb in probs:
        pb["K_que"] = H.rand_storage((pb["n_que"], 128), torch.bfloat16, gen)
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    loop = ChunkLoop(fin, probs, w.chunk, history=True)
    loop.run()
    st = H.validate_chunk_loop(loop, [0, 1, 2, 3], "C4 exact denominator")
    say(f"  {st}")
    fin.close()
