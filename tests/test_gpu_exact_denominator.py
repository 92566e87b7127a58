"""GPU parity of the paper-exact softmax denominator: the per-row term of the prompt's
own (causal) keys from finch_prompt_lse, and scoring / selection with it."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

SPECS = [
    dict(n_que=48, c=300, m=1000, r=200, prompt_keys=True),
    dict(n_que=1, c=0, m=257, r=17, prompt_keys=True),
    dict(n_que=5, c=37, m=255, r=100, prompt_keys=True),
    dict(n_que=16, c=64, m=0, r=10, prompt_keys=True),
    dict(n_que=33, c=511, m=513, r=512, prompt_keys=True),
    dict(n_que=7, c=1, m=2047, r=1024, prompt_keys=True, qscale=3.0),
]


def say(msg):
    print(msg, flush=True)


def check_prompt_lse(ts, group, what):
    worst = 0.0
    for t in ts:
        want = O.prompt_lse(W.to_numpy_storage(t["q"]), W.to_numpy_storage(t["k_que"]), group)
        got = t["lse_extra"][:-1].double().cpu().numpy()
        err = np.abs(got - want).max()
        assert err < 1e-5 * max(1.0, np.abs(want).max()), f"{what}: lse_extra off by {err:.3e}"
        assert float(t["lse_extra"][-1]) == -77.0
        worst = max(worst, err)
    return worst


@pytest.mark.parametrize("dtype,d,group,path", [
    (torch.bfloat16, 128, 4, "separate"), (torch.bfloat16, 128, 4, "owner"), (torch.bfloat16, 64, 1, "separate"),
    (torch.bfloat16, 64, 2, "owner"), (torch.float32, 64, 1, "separate"), (torch.float32, 128, 2, "separate")])
def test_scores_with_the_prompts_own_keys_in_the_denominator(dtype, d, group, path):
    say(f"exact denominator {dtype} d={d} G={group} {path}")
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    fin.set_step_path({"separate": F.FINCH_PATH_SEPARATE, "owner": F.FINCH_PATH_OWNER}[path])
    specs = SPECS if dtype == torch.bfloat16 else [dict(s, n_que=min(s["n_que"], 24)) for s in SPECS]
    batch, ts = H.single_step_case(fin, specs, dtype, d, group, seed=700 + d + group)
    fin.prompt_lse(batch)
    torch.cuda.synchronize()
    say(f"  worst lse_extra error {check_prompt_lse(ts, group, 'prompt_lse'):.2e}")
    fin.step(batch)
    st = H.validate_single_step(ts, f"exact {path}")
    say(f"  worst score rel err {st['worst_rel']:.2e}, swaps {st['swaps']}")
    for t in ts:
        N, R = t["c"] + t["m"], group * t["n_que"]
        total = float(t["scores"][:N].double().sum())
        assert 0.0 < total < R, (total, R)      # the prompt keeps its share of every row
    fin.close()


def test_many_slices_and_the_separate_scoring_call():
    """More than 16 slices (the statistics are merged by their own kernel) and
    finch_score on its own, both with the widened denominator."""
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_SLICE_KEYS, 256)
    specs = [dict(n_que=40, c=1000, m=4200, r=333, prompt_keys=True), dict(n_que=3, c=0, m=290, r=20, prompt_keys=True)]
    b1, t1 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=13)
    b2, t2 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=13)
    fin.prompt_lse(b1); fin.prompt_lse(b2)
    fin.step(b1)
    H.validate_single_step(t1, "exact, 20 slices")
    fin.score(b2); fin.topk(b2); fin.compact(b2)
    torch.cuda.synchronize()
    for a, b in zip(t1, t2):
        for name in ("scores", "idx", "k_out", "v_out"):
            assert torch.equal(a[name], b[name]), name
    fin.close()


@pytest.mark.parametrize("path", ["owner", "separate"])
def test_chunk_loop_with_exact_denominator(path):
    """The whole loop (one launch with one workgroup per problem, or step by step) with
    the prompt's own keys in every denominator; a per-step prompt for one problem."""
    from paper_2408_00167_amd.driver import ChunkLoop
    say(f"exact denominator loop {path}")
    w = W.get_workload("C4")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path({"separate": F.FINCH_PATH_SEPARATE, "owner": F.FINCH_PATH_OWNER}[path])
    gen = torch.Generator(device="cuda"); gen.manual_seed(31)
    probs = []
    for j, n in enumerate([2048, 1300, 2048]):
        pb = H.make_gpu_problem(w, 0, 0, j, n_cont=n)
        pb["budget"] = n // 8
        steps = (n + 511) // 512
        if j == 1:
            pb["Q"] = [H.rand_storage(tuple(pb["Q"].shape), torch.bfloat16, gen) for _ in range(steps)]
            pb["K_que"] = [H.rand_storage((pb["n_que"], 128), torch.bfloat16, gen) for _ in range(steps)]
        else:
            pb["K_que"] = H.rand_storage((pb["n_que"], 128), torch.bfloat16, gen)
        probs.append(pb)
    loop = ChunkLoop(fin, probs, 512, history=True)
    loop.run()
    st = H.validate_chunk_loop(loop, [0, 1, 2], f"exact loop {path}")
    say(f"  {st}")
    fin.close()


def test_prompt_lse_argument_checks():
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    batch, ts = H.single_step_case(fin, [dict(n_que=4, c=0, m=64, r=8)], torch.bfloat16, 128, 4, seed=1)
    with pytest.raises(F.FinchError) as e:      # no k_que, no lse_extra
        fin.prompt_lse(batch)
    assert e.value.status == F.FINCH_ERR_INVALID_ARG
    fin.close()
