"""Seeded sweep over problem shapes: batches of random (n_que, c, m, r) with the
degenerate values mixed in (no cache, no chunk, keep nothing, keep everything, one
candidate), both dtypes, every group size and both launch paths, with and without the
optional inputs (document rows, the prompt's own keys), each problem against the
oracle.  Complements the hand-picked cases of the other GPU tests."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _specs(rng, bf16: bool, options: bool, trial: int):
    specs = []
    for _ in range(int(rng.integers(1, 6))):
        n_que = int(rng.integers(1, 70 if bf16 else 20))
        c = int(rng.choice([0, 0, int(rng.integers(1, 700))]))
        m = int(rng.choice([0, 1, int(rng.integers(1, 1500)), int(rng.integers(200, 2500))]))
        if c + m == 0:
            m = 5
        r = int(rng.choice([0, 1, c + m, c + m + 3, int(rng.integers(1, c + m + 1))]))
        sp = dict(n_que=n_que, c=c, m=m, r=r)
        if rng.random() < 0.2:
            sp["qscale"] = float(rng.choice([0.1, 3.0, 6.0]))
        if options and bf16:
            if rng.random() < 0.5 and m > 0:
                sp["doc_rows"] = True
                sp["m"] = m = min(m, 500)
                sp["r"] = min(sp["r"], c + m + 3)
                if trial % 2 == 1 and rng.random() < 0.3:
                    sp["no_prompt"] = True
            if trial % 2 == 0:
                sp["prompt_keys"] = True
        specs.append(sp)
    return specs


@pytest.mark.parametrize("seed,options", [(11, False), (12, False), (13, True)])
def test_random_shapes(seed, options):
    rng = np.random.default_rng(seed)
    problems = 0
    for trial in range(9):
        bf16 = options or trial % 3 != 0
        dtype = torch.bfloat16 if bf16 else torch.float32
        d = int(rng.choice([64, 128]))
        group = int(rng.choice([1, 2, 4, 8]))
        path = ["auto", "separate", "owner"][trial % 3] if bf16 else "auto"
        specs = _specs(rng, bf16, options, trial)
        with_doc = any(sp.get("doc_rows") for sp in specs)
        say(f"seed {seed} trial {trial}: {dtype} d={d} G={group} path={path} {specs}")
        fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
        if bf16 and path != "auto" and not with_doc:
            fin.set_step_path(dict(separate=F.FINCH_PATH_SEPARATE, owner=F.FINCH_PATH_OWNER)[path])
        batch, ts = H.single_step_case(fin, specs, dtype, d, group, seed=1000 * seed + trial)
        if any(sp.get("prompt_keys") for sp in specs):
            fin.prompt_lse(batch)
        fin.step(batch)
        st = H.validate_single_step(ts, f"sweep seed {seed} trial {trial}")
        say(f"   worst score rel err {st['worst_rel']:.2e}, near-tie swaps {st['swaps']}")
        fin.close()
        problems += len(specs)
    say(f"seed {seed}: {problems} problems")


@pytest.mark.parametrize("seed", [21, 22])
def test_random_chunk_loops(seed):
    """Whole chunk loops with random document lengths, chunk sizes, prompt lengths and
    budgets (so that the cache grows through several key blocks and the slots drop out
    at different steps), as one launch and step by step, every step against the oracle."""
    import workloads as W
    from paper_2408_00167_amd.driver import ChunkLoop
    rng = np.random.default_rng(seed)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    for trial in range(3):
        d = int(rng.choice([64, 128]))
        group = int(rng.choice([1, 4]))
        chunk = int(rng.choice([96, 256, 700]))
        fin = F.Finch(F.FINCH_BF16, d, group)
        fin.set_step_path([F.FINCH_PATH_AUTO, F.FINCH_PATH_OWNER, F.FINCH_PATH_SEPARATE][trial])
        probs = []
        for j in range(int(rng.integers(2, 6))):
            n = int(rng.integers(chunk // 2, 9 * chunk))
            n_que = int(rng.integers(1, 50))
            probs.append(dict(Q=H.rand_storage((group * n_que, d), torch.bfloat16, gen),
                              K=H.rand_storage((n, d), torch.bfloat16, gen),
                              V=H.rand_storage((n, d), torch.bfloat16, gen),
                              n_que=n_que, budget=int(rng.integers(1, max(2, n // 2))), id=j))
        say(f"seed {seed} trial {trial}: d={d} G={group} chunk={chunk} "
            f"lengths={[int(p['K'].shape[0]) for p in probs]} budgets={[p['budget'] for p in probs]}")
        outs = []
        for per_step in (False, True):
            loop = ChunkLoop(fin, probs, chunk, history=True)
            loop.run(per_step=per_step)
            st = H.validate_chunk_loop(loop, list(range(len(probs))), f"sweep loop per_step={per_step}")
            say(f"   per_step={per_step}: {st}")
            outs.append(loop)
        assert torch.equal(outs[0].idx, outs[1].idx)
        fin.close()
