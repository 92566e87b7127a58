"""GPU parity of the re-positioned compaction (kept keys rotated to their new
slots, ascending or rank order) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

PAIRING = {"half": F.FINCH_ROPE_HALF, "interleaved": F.FINCH_ROPE_INTERLEAVED, None: F.FINCH_ROPE_OFF}
ORDER = {"ascending": F.FINCH_ORDER_ASCENDING, "rank": F.FINCH_ORDER_RANK}

SPECS = [
    dict(n_que=24, c=300, m=1000, r=200),
    dict(n_que=1, c=0, m=257, r=17),
    dict(n_que=5, c=37, m=255, r=100),
    dict(n_que=16, c=64, m=0, r=10),          # cache-only step
    dict(n_que=16, c=0, m=1, r=1),
    dict(n_que=16, c=100, m=156, r=0),        # keep nothing
    dict(n_que=16, c=100, m=156, r=256),      # keep everything: no key moves (ascending)
    dict(n_que=7, c=1, m=2047, r=1024),
    dict(n_que=3, c=65, m=70, r=65),          # one row past a 64-row workgroup
]


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("order", ["ascending", "rank"])
@pytest.mark.parametrize("pairing", ["half", "interleaved", None])
@pytest.mark.parametrize("dtype,d,group", [(torch.bfloat16, 128, 4), (torch.bfloat16, 64, 1),
                                           (torch.float32, 64, 1), (torch.float32, 128, 2)])
def test_step_with_repositioning(dtype, d, group, pairing, order):
    if pairing is None and order == "ascending":
        pytest.skip("the plain copy is covered by the parity tests")
    base = 10000.0 if d == 128 else 500000.0
    say(f"reposition {dtype} d={d} G={group} pairing={pairing} order={order}")
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    fin.set_reposition(PAIRING[pairing], ORDER[order], base)
    batch, ts = H.single_step_case(fin, SPECS, dtype, d, group, seed=500 + d + group)
    fin.step(batch)
    st = H.validate_single_step(ts, f"repos {pairing}/{order}", repos=(pairing, order, base))
    say(f"  worst rotation error / row max {st['worst_rot']:.2e}, swaps {st['swaps']}")
    # keep everything in ascending order: every shift is 0, the copy is bit-exact
    if order == "ascending":
        t = ts[6]
        both = torch.cat([t["k_cache"], t["k_chunk"]])
        assert torch.equal(t["k_out"][:256], both)
    # back to plain copies on the same context
    fin.set_reposition()
    for t in ts:
        t["k_out"].fill_(7.0); t["v_out"].fill_(7.0); t["idx"].fill_(-9); t["scores"].fill_(-5.0)
    fin.step(batch)
    H.validate_single_step(ts, "plain again")
    fin.close()


@pytest.mark.parametrize("order", ["ascending", "rank"])
@pytest.mark.parametrize("pairing", ["half", "interleaved", None])
@pytest.mark.parametrize("d,group", [(128, 4), (64, 2)])
def test_one_workgroup_per_problem_repositions(d, group, pairing, order):
    if pairing is None and order == "ascending":
        pytest.skip("the plain copy is covered by the parity tests")
    say(f"reposition owner d={d} G={group} {pairing} {order}")
    fin = F.Finch(F.FINCH_BF16, d, group)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    fin.set_reposition(PAIRING[pairing], ORDER[order], 10000.0)
    batch, ts = H.single_step_case(fin, SPECS, torch.bfloat16, d, group, seed=600 + d)
    fin.step(batch)
    st = H.validate_single_step(ts, f"owner repos {pairing} {order}", repos=(pairing, order, 10000.0))
    say(f"  worst rotation error / row max {st['worst_rot']:.2e}")
    # the per-stage kernels give the same bits
    fin.set_step_path(F.FINCH_PATH_SEPARATE)
    b2, t2 = H.single_step_case(fin, SPECS, torch.bfloat16, d, group, seed=600 + d)
    fin.step(b2)
    torch.cuda.synchronize()
    for a, b in zip(ts, t2):
        assert torch.equal(a["idx"], b["idx"])
        # (slots by rank follow each path's own fp32 scores, whose last bits may differ
        # between the paths: both are checked against the oracle, each with its scores)
        if order == "ascending":
            assert torch.equal(a["k_out"], b["k_out"]) and torch.equal(a["v_out"], b["v_out"])
    if order == "rank":
        H.validate_single_step(t2, f"per-stage repos {pairing} rank", repos=(pairing, order, 10000.0))
    fin.close()


@pytest.mark.parametrize("order", ["ascending", "rank"])
def test_whole_loop_with_repositioning_equals_step_by_step(order):
    from paper_2408_00167_amd.driver import ChunkLoop
    w = W.get_workload("C4")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    fin.set_reposition(F.FINCH_ROPE_HALF, ORDER[order], 500000.0)
    probs = []
    for j, n in enumerate([2048, 1300, 1800]):
        pb = H.make_gpu_problem(w, 0, 0, j, n_cont=n)
        pb["budget"] = n // 6
        probs.append(pb)
    finals = []
    for per_step in (False, True):
        loop = ChunkLoop(fin, probs, 512, history=True)
        loop.run(per_step=per_step)
        torch.cuda.synchronize()
        finals.append([tuple(t.clone() for t in loop.final_cache(p)) for p in range(len(probs))] + [loop.idx.clone()])
    for a, b in zip(finals[0][:-1], finals[1][:-1]):
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert torch.equal(finals[0][-1], finals[1][-1])
    fin.close()


def test_shifts_of_hundreds_of_thousands_of_positions():
    """One long chunk: kept keys move up to 3*10^5 positions towards the start, so the
    angle must be reduced before sine and cosine are taken."""
    say("reposition far")
    fin = F.Finch(F.FINCH_BF16, 128, 1)
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_ASCENDING, 10000.0)
    batch, ts = H.single_step_case(fin, [dict(n_que=8, c=0, m=300000, r=48)], torch.bfloat16, 128, 1, seed=77)
    fin.step(batch)
    torch.cuda.synchronize()
    t = ts[0]
    idx = t["idx"].cpu().numpy()[:48]
    assert (np.diff(idx) > 0).all() and idx.max() > 100000
    Kk = W.to_numpy_storage(t["k_chunk"])
    Vk = W.to_numpy_storage(t["v_chunk"])
    err = H.check_repositioned(t, Kk[:0], Kk, Vk[:0], Vk, idx, 48, "half", "ascending", 10000.0, "far")
    say(f"  worst rotation error / row max {err:.2e}")
    fin.close()


def test_separate_compact_call_and_argument_checks():
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    specs = [dict(n_que=12, c=40, m=300, r=64), dict(n_que=4, c=0, m=90, r=33)]
    b1, t1 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=8)
    b2, t2 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=8)
    fin.set_reposition(F.FINCH_ROPE_INTERLEAVED, F.FINCH_ORDER_RANK, 1e6)
    fin.step(b1)
    fin.score(b2); fin.topk(b2); fin.compact(b2)
    torch.cuda.synchronize()
    for a, b in zip(t1, t2):
        for name in ("scores", "idx", "k_out", "v_out"):
            assert torch.equal(a[name], b[name]), name
    # rank order needs the scores in finch_compact
    b3, t3 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=8, null_scores=True)
    with pytest.raises(F.FinchError) as e:
        fin.compact(b3)
    assert e.value.status == F.FINCH_ERR_INVALID_ARG
    fin.step(b3)    # finch_step keeps them in the workspace
    torch.cuda.synchronize()
    for a, b in zip(t1, t3):
        assert torch.equal(a["k_out"], b["k_out"]) and torch.equal(a["v_out"], b["v_out"])
    # one workgroup per problem ranks its kept rows in LDS: up to 2048 of them
    fin.set_step_path(F.FINCH_PATH_OWNER)
    big, _ = H.single_step_case(fin, [dict(n_que=4, c=0, m=3000, r=2049)], torch.bfloat16, 128, 4, seed=8)
    with pytest.raises(F.FinchError) as e:
        fin.step(big)
    assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    fin.set_step_path(F.FINCH_PATH_AUTO)
    for bad in (dict(pairing=7), dict(order=5), dict(pairing=F.FINCH_ROPE_HALF, base=0.5)):
        with pytest.raises(F.FinchError) as e:
            fin.set_reposition(**bad)
        assert e.value.status == F.FINCH_ERR_INVALID_ARG
    fin.close()


def test_chunk_loop_with_repositioned_cache():
    """Three steps by hand: the cache a step produces (rotated keys, rank order) is the
    next step's input; every step is checked against the oracle on the GPU's own inputs."""
    say("reposition loop")
    d, G, m, base = 128, 4, 600, 10000.0
    fin = F.Finch(F.FINCH_BF16, d, G)
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_RANK, base)
    gen = torch.Generator(device="cuda"); gen.manual_seed(99)
    q = H.rand_storage((G * 10, d), torch.bfloat16, gen)
    doc_k = H.rand_storage((3 * m, d), torch.bfloat16, gen)
    doc_v = H.rand_storage((3 * m, d), torch.bfloat16, gen)
    kc = torch.empty(0, d, dtype=torch.bfloat16, device="cuda")
    vc = torch.empty(0, d, dtype=torch.bfloat16, device="cuda")
    for i, r in enumerate((150, 300, 450)):
        t = dict(q=q, k_cache=kc, v_cache=vc, k_chunk=doc_k[i * m:(i + 1) * m], v_chunk=doc_v[i * m:(i + 1) * m],
                 k_out=torch.full((r, d), 7.0, device="cuda").to(torch.bfloat16),
                 v_out=torch.full((r, d), 7.0, device="cuda").to(torch.bfloat16),
                 scores=torch.empty(kc.shape[0] + m, device="cuda"),
                 idx=torch.empty(r, dtype=torch.int32, device="cuda"), n_que=10, c=kc.shape[0], m=m, r=r)
        fin.step(F.Batch([t]))
        torch.cuda.synchronize()
        Kc, Kk = W.to_numpy_storage(kc), W.to_numpy_storage(t["k_chunk"])
        Vc, Vk = W.to_numpy_storage(vc), W.to_numpy_storage(t["v_chunk"])
        want = O.key_scores(W.to_numpy_storage(q), Kc, Kk)
        H.check_scores(t["scores"].cpu().numpy(), want, H.SCORE_TOL["bf16"], f"step {i}")
        idx = t["idx"].cpu().numpy()
        H.check_indices(idx, want, r, f"step {i}")
        H.check_repositioned(t, Kc, Kk, Vc, Vk, idx, r, "half", "rank", base, f"step {i}")
        kc, vc = t["k_out"], t["v_out"]
    fin.close()
