"""GPU parity of the conditioning on the chunk's own rows (the paper's ablation:
document-only or document + prompt self-attention with the causal mask and the
normalisation step) against the oracle."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

SPECS = [
    dict(n_que=24, c=300, m=700, r=200, doc_rows=True),                  # three row chunks per head
    dict(n_que=5, c=37, m=255, r=100, doc_rows=True),
    dict(n_que=1, c=0, m=257, r=17, doc_rows=True),                      # first chunk: no cache
    dict(n_que=16, c=64, m=0, r=10, doc_rows=True),                      # cache-only step: no document rows
    dict(n_que=16, c=0, m=1, r=1, doc_rows=True),
    dict(n_que=8, c=100, m=156, r=256, doc_rows=True),
    dict(n_que=40, c=900, m=40, r=64, doc_rows=True, prompt_keys=True),  # with the prompt's own keys as well
    dict(n_que=3, c=5, m=600, r=77, doc_rows=True, no_prompt=True),      # document rows only
    dict(n_que=3, c=0, m=33, r=20, doc_rows=True, no_prompt=True),
]


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("d,group", [(128, 4), (64, 1), (128, 1), (64, 3)])
def test_document_rows_with_causal_mask(d, group, dtype):
    say(f"conditioning d={d} G={group} {dtype}")
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    specs = SPECS if dtype == torch.bfloat16 else [dict(sp, m=min(sp["m"], 300), c=min(sp["c"], 200)) for sp in SPECS]
    batch, ts = H.single_step_case(fin, specs, dtype, d, group, seed=1100 + d + group)
    with_keys = F.Batch([t for t in batch_descs(ts) if t.get("k_que") is not None])
    fin.prompt_lse(with_keys)
    fin.step(batch)
    st = H.validate_single_step(ts, f"conditioning d={d} G={group}")
    say(f"  worst score rel err {st['worst_rel']:.2e}, swaps {st['swaps']}")
    for t in ts:     # every score is the sum of the row weights: prompt rows 1, document row i (c+i+1)/(c+m)
        c, m = t["c"], t["m"]
        N = c + m
        if t.get("lse_extra") is not None or N == 0:
            continue
        rows_p = 0 if t["q"] is None else group * t["n_que"]
        want = rows_p + group * sum((c + i + 1) / N for i in range(m)) * (t.get("q_doc") is not None)
        got = float(t["scores"][:N].double().sum())
        assert abs(got - want) < 1e-3 * max(1.0, want), (got, want)
    ran = profile_kernels(fin, batch)
    assert ran == {"owner"}, ran
    fin.close()


def batch_descs(ts):
    out = []
    for t in ts:
        d = dict(t)
        if t.get("lse_extra") is not None:
            d["lse_extra"] = t["lse_extra"][:-1]
        out.append(d)
    return out


def profile_kernels(fin, batch):
    F.finch_profile(fin.ctx, True)
    fin.step(batch)
    torch.cuda.synchronize()
    prof = F.finch_profile_read(fin.ctx)
    F.finch_profile(fin.ctx, False)
    return {k for k, v in prof.items() if v["launches"]}


def test_whole_loop_call_and_separate_scoring_call():
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    specs = [s for s in SPECS if not s.get("prompt_keys")]
    b1, t1 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=1200)
    b2, t2 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=1200)
    b3, t3 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=1200)
    fin.step(b1)
    fin.score(b2); fin.topk(b2); fin.compact(b2)
    # single_step_case hands exactly-sized views to its own Batch; do the same here
    lb_descs = batch_descs(t3)
    for dsc, t in zip(lb_descs, t3):
        N, rr = t["c"] + t["m"], min(t["r"], t["c"] + t["m"])
        dsc["k_out"], dsc["v_out"], dsc["idx"] = t["k_out"][:max(rr, 1)], t["v_out"][:max(rr, 1)], t["idx"][:max(rr, 1)]
        dsc["scores"] = t["scores"][:max(N, 1)]
    lb = F.LoopBatch([lb_descs])
    fin.loop(lb)
    torch.cuda.synchronize()
    for a, b, c in zip(t1, t2, t3):
        for name in ("scores", "idx", "k_out", "v_out"):
            assert torch.equal(a[name], b[name]), name
            assert torch.equal(a[name], c[name]), name
    H.validate_single_step(t3, "conditioning, loop call")
    fin.close()


def test_chunk_loop_with_document_rows():
    """The whole loop in one launch, every step of every problem against the oracle;
    a ragged last chunk and a per-step set of document rows for one problem."""
    from paper_2408_00167_amd.driver import ChunkLoop
    w = W.get_workload("C4")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    gen = torch.Generator(device="cuda"); gen.manual_seed(41)
    probs = []
    for j, n in enumerate([1536, 1300, 900]):
        pb = H.make_gpu_problem(w, 0, 0, j, n_cont=n)
        pb["budget"] = n // 6
        steps = (n + 511) // 512
        mk = lambda: H.rand_storage((4 * 512, 128), torch.bfloat16, gen).reshape(4, 512, 128)
        pb["Q_doc"] = [mk() for _ in range(steps)] if j == 1 else mk()
        probs.append(pb)
    for per_step in (False, True):
        loop = ChunkLoop(fin, probs, 512, history=True)
        loop.run(per_step=per_step)
        st = H.validate_chunk_loop(loop, [0, 1, 2], f"document rows, per_step={per_step}")
        say(f"  per_step={per_step}: {st}")
    fin.close()


def test_paths_without_those_rows_refuse():
    sp = [dict(n_que=4, c=0, m=64, r=8, doc_rows=True)]
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    batch, ts = H.single_step_case(fin, sp, torch.bfloat16, 128, 4, seed=4)
    fin.set_step_path(F.FINCH_PATH_SEPARATE)
    for call in (fin.step, fin.score):
        with pytest.raises(F.FinchError) as e:
            call(batch)
        assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    fin.set_step_path(F.FINCH_PATH_AUTO)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 1)
    fin.step(batch)
    H.validate_single_step(ts, "after the refused calls")
    fin.close()
    # fp32: the same rule (rows of the chunk's own tokens only with one workgroup per problem)
    f32 = F.Finch(F.FINCH_F32, 64, 1)
    batch, ts = H.single_step_case(f32, sp, torch.float32, 64, 1, seed=4)
    f32.set_step_path(F.FINCH_PATH_SEPARATE)
    with pytest.raises(F.FinchError) as e:
        f32.step(batch)
    assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    f32.set_step_path(F.FINCH_PATH_AUTO)
    f32.step(batch)
    H.validate_single_step(ts, "fp32 document rows")
    f32.close()
