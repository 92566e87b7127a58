"""GPU parity of the paper's layer-wise selection: the scores of all KV heads of a
layer are summed and one index set serves every head."""
import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
import workloads as W
from oracle import finch_oracle as O
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

LAYERS = [
    dict(n_que=24, c=300, m=1000, r=200),
    dict(n_que=5, c=37, m=255, r=100),
    dict(n_que=16, c=64, m=0, r=10),
    dict(n_que=16, c=100, m=156, r=0),
    dict(n_que=16, c=100, m=156, r=256),      # keep everything
    dict(n_que=3, c=0, m=17000, r=700),       # more candidates than the register select holds
]


def say(msg):
    print(msg, flush=True)


def validate_layers(ts, L, what):
    torch.cuda.synchronize()
    swaps = 0
    for run in range(len(ts) // L):
        heads = ts[run * L:(run + 1) * L]
        t0 = heads[0]
        N, r = t0["c"] + t0["m"], t0["r"]
        rr = min(r, N)
        per_head = []
        for t in heads:
            want = O.key_scores(W.to_numpy_storage(t["q"]), W.to_numpy_storage(t["k_cache"]),
                                W.to_numpy_storage(t["k_chunk"]))
            H.check_scores(t["scores"].cpu().numpy()[:N], want, H.SCORE_TOL[H.dtype_name(t["k_out"])], f"{what} run {run}")
            per_head.append(want)
        total = O.layer_scores(per_head)
        idx = t0["idx"].cpu().numpy()
        swaps += H.check_indices(idx[:rr], total, r, f"{what} run {run}")
        # the decision itself, in the precision the GPU takes it in: fp32 sums, head by head
        acc = heads[0]["scores"].cpu().numpy()[:N].copy()
        for t in heads[1:]:
            acc = acc + t["scores"].cpu().numpy()[:N]
        assert idx[:rr].tolist() == O.top_r(acc, r).tolist(), f"{what} run {run}: not the top r of the fp32 sums"
        for t in heads:
            assert torch.equal(t["idx"], t0["idx"]), f"{what} run {run}: heads disagree"
            Kc, Kk = W.to_numpy_storage(t["k_cache"]), W.to_numpy_storage(t["k_chunk"])
            Vc, Vk = W.to_numpy_storage(t["v_cache"]), W.to_numpy_storage(t["v_chunk"])
            assert W.to_numpy_storage(t["k_out"])[:rr].tobytes() == O.gather_rows(idx[:rr], Kc, Kk).tobytes()
            assert W.to_numpy_storage(t["v_out"])[:rr].tobytes() == O.gather_rows(idx[:rr], Vc, Vk).tobytes()
            assert int(t["idx"][max(rr, 1)]) == -9
    return swaps


@pytest.mark.parametrize("dtype,d,group,L,path", [(torch.bfloat16, 128, 4, 8, "separate"), (torch.bfloat16, 64, 1, 3, "separate"),
                                                  (torch.float32, 64, 1, 2, "separate"),
                                                  (torch.bfloat16, 128, 4, 8, "owner"), (torch.bfloat16, 64, 1, 3, "owner"),
                                                  (torch.bfloat16, 128, 2, 16, "owner")])
def test_layer_wise_selection(dtype, d, group, L, path):
    """One kernel per stage (the layer's scores summed by the selection kernel), or one
    workgroup per problem (the L workgroups of a layer wait for each other's scores)."""
    say(f"layer-wise {dtype} d={d} G={group} L={L} {path}")
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    fin.set_step_path(F.FINCH_PATH_OWNER if path == "owner" else F.FINCH_PATH_SEPARATE)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, L)
    layers = LAYERS if dtype == torch.bfloat16 else [dict(s, n_que=min(s["n_que"], 8), m=min(s["m"], 1200)) for s in LAYERS]
    specs = [sp for sp in layers for _ in range(L)]
    b1, t1 = H.single_step_case(fin, specs, dtype, d, group, seed=900 + L)
    fin.step(b1)
    say(f"  swaps {validate_layers(t1, L, 'step')}")
    assert fin.workspace_status() == 0
    b2, t2 = H.single_step_case(fin, specs, dtype, d, group, seed=900 + L)
    fin.score(b2); fin.topk(b2); fin.compact(b2)      # (top-r and compaction alone always run per stage)
    torch.cuda.synchronize()
    for a, b in zip(t1, t2):
        for name in ("scores", "idx", "k_out", "v_out"):
            assert torch.equal(a[name], b[name]), name
    # the scores may stay in the workspace
    b3, t3 = H.single_step_case(fin, specs, dtype, d, group, seed=900 + L, null_scores=True)
    fin.step(b3)
    torch.cuda.synchronize()
    for a, b in zip(t1, t3):
        assert torch.equal(a["idx"], b["idx"]) and torch.equal(a["k_out"], b["k_out"])
    fin.close()


@pytest.mark.parametrize("dtype,d,group,L,path", [(torch.bfloat16, 128, 4, 8, "owner"), (torch.bfloat16, 128, 4, 8, "separate"),
                                                  (torch.bfloat16, 64, 2, 4, "owner"), (torch.float32, 64, 1, 2, "owner"),
                                                  (torch.float32, 64, 1, 2, "separate")])
def test_the_papers_own_configuration(dtype, d, group, L, path):
    """The options together, as the paper words the method: the prompt's own keys in the
    denominator, the scores summed over the heads of a layer and one top-r per layer, kept keys
    re-positioned (ascending slots) while they are compacted."""
    say(f"paper-literal {dtype} d={d} G={group} L={L} {path}")
    base = 10000.0
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    fin.set_step_path(F.FINCH_PATH_OWNER if path == "owner" else F.FINCH_PATH_SEPARATE)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, L)
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_ASCENDING, base)
    layers = [dict(n_que=24, c=300, m=1000, r=200), dict(n_que=5, c=37, m=255, r=100),
              dict(n_que=16, c=100, m=156, r=256), dict(n_que=9, c=0, m=700, r=33)]
    if dtype == torch.float32:
        layers = [dict(sp, n_que=min(sp["n_que"], 8)) for sp in layers]
    specs = [dict(sp, prompt_keys=True) for sp in layers for _ in range(L)]
    batch, ts = H.single_step_case(fin, specs, dtype, d, group, seed=4242 + L)
    fin.prompt_lse(batch)
    fin.step(batch)
    torch.cuda.synchronize()
    assert fin.workspace_status() == 0
    tol = H.SCORE_TOL[H.dtype_name(ts[0]["k_out"])]
    swaps, worst_rot = 0, 0.0
    for run in range(len(ts) // L):
        heads = ts[run * L:(run + 1) * L]
        t0 = heads[0]
        N, r = t0["c"] + t0["m"], t0["r"]
        rr = min(r, N)
        per_head = []
        for t in heads:
            want_extra = O.prompt_lse(W.to_numpy_storage(t["q"]), W.to_numpy_storage(t["k_que"]), group)
            extra = t["lse_extra"][:-1].double().cpu().numpy()
            assert np.abs(extra - want_extra).max() < 1e-5 * max(1.0, np.abs(want_extra).max())
            # (the scoring is checked with the term the GPU was given, itself checked just above)
            want = O.key_scores(W.to_numpy_storage(t["q"]), W.to_numpy_storage(t["k_cache"]),
                                W.to_numpy_storage(t["k_chunk"]), lse_extra=extra)
            H.check_scores(t["scores"].cpu().numpy()[:N], want, tol, f"run {run}")
            per_head.append(want)
        idx = t0["idx"].cpu().numpy()
        swaps += H.check_indices(idx[:rr], O.layer_scores(per_head), r, f"run {run}")
        for t in heads:
            assert torch.equal(t["idx"], t0["idx"]), f"run {run}: heads disagree"
            Kc, Kk = W.to_numpy_storage(t["k_cache"]), W.to_numpy_storage(t["k_chunk"])
            Vc, Vk = W.to_numpy_storage(t["v_cache"]), W.to_numpy_storage(t["v_chunk"])
            worst_rot = max(worst_rot, H.check_repositioned(t, Kc, Kk, Vc, Vk, idx, rr, "half", "ascending", base,
                                                            f"run {run}"))
    say(f"  swaps {swaps}, worst rotation error / row max {worst_rot:.2e}")
    fin.close()


def test_a_wait_that_expires_is_reported():
    """The bound on a workgroup's wait for its layer, forced from the host: with a bound of 0
    ticks the first workgroup of a layer to arrive gives up at once and leaves its indices
    unwritten, the launch still runs to its end, and finch_workspace_status reports it; with
    the default bound the same batch runs clean again."""
    say("layer wait bound")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 8)
    specs = [sp for sp in LAYERS for _ in range(8)]
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_WAIT_TICKS, 0)
    b0, t0 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=77)
    fin.step(b0)
    with pytest.raises(F.FinchError) as e:
        fin.workspace_status()
    assert e.value.status == F.FINCH_ERR_TIMEOUT
    untouched = 0
    for t in t0:   # a workgroup that gave up wrote no indices; the others wrote theirs inside the buffer
        rr = min(t["r"], t["c"] + t["m"])
        idx = t["idx"][:rr].cpu().numpy()
        if rr and (idx == -9).all():
            untouched += 1
        else:
            assert ((idx >= 0) & (idx < t["c"] + t["m"])).all()
        assert int(t["idx"][max(rr, 1)]) == -9
    assert untouched >= 1
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_WAIT_TICKS, 20_000_000)
    b1, t1 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=77)
    fin.step(b1)
    assert fin.workspace_status() == 0
    say(f"  swaps {validate_layers(t1, 8, 'after the bound was restored')}")
    with pytest.raises(F.FinchError):
        F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_WAIT_TICKS, -1)
    fin.close()


def test_layer_group_argument_checks():
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 2)
    sp = dict(n_que=4, c=0, m=64, r=8)
    for specs in ([sp] * 3, [sp, dict(sp, r=9)], [sp, dict(sp, m=65)]):
        batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=2)
        with pytest.raises(F.FinchError) as e:
            fin.step(batch)
        assert e.value.status == F.FINCH_ERR_INVALID_ARG
    batch, ts = H.single_step_case(fin, [sp] * 4, torch.bfloat16, 128, 4, seed=2)
    # one workgroup per problem: only while a layer's workgroups fit on the chip together
    # and the layer has at most 16 heads
    fin.set_step_path(F.FINCH_PATH_OWNER)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 32)
    b32, _ = H.single_step_case(fin, [sp] * 32, torch.bfloat16, 128, 4, seed=2)
    with pytest.raises(F.FinchError) as e:
        fin.step(b32)
    assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 2)
    many, _ = H.single_step_case(fin, [sp] * 600, torch.bfloat16, 128, 4, seed=2)
    with pytest.raises(F.FinchError) as e:
        fin.step(many)
    assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    fin.set_step_path(F.FINCH_PATH_AUTO)
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_RANK, 1e4)
    with pytest.raises(F.FinchError) as e:
        fin.step(batch)
    assert e.value.status == F.FINCH_ERR_UNSUPPORTED
    fin.set_reposition(F.FINCH_ROPE_HALF, F.FINCH_ORDER_ASCENDING, 1e4)
    fin.step(batch)      # rotation with ascending slots goes together with layer groups
    torch.cuda.synchronize()
    assert torch.equal(ts[0]["idx"], ts[1]["idx"]) and torch.equal(ts[2]["idx"], ts[3]["idx"])
    with pytest.raises(F.FinchError):
        F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 0)
    fin.close()
