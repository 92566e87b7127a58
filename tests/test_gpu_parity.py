"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on
the same seeded inputs.  Every test here needs a real MI355X."""
import ctypes

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


# --------------------------------------------------------------- single steps

RAGGED_SPECS = [
    dict(n_que=48, c=300, m=1000, r=200),     # 6 tiles, ragged tail
    dict(n_que=1, c=0, m=257, r=17),          # one prompt row per head, first chunk
    dict(n_que=5, c=37, m=255, r=100),        # R not a multiple of 32
    dict(n_que=128, c=64, m=0, r=10),         # cache-only step (m = 0), R = 512
    dict(n_que=16, c=0, m=1, r=1),            # a single candidate
    dict(n_que=16, c=100, m=156, r=0),        # keep nothing
    dict(n_que=16, c=100, m=156, r=256),      # keep everything (identity)
    dict(n_que=16, c=100, m=156, r=1000),     # r above N is clamped
    dict(n_que=33, c=511, m=513, r=512),      # exactly 4 tiles
    dict(n_que=7, c=1, m=2047, r=1024),
]


@pytest.mark.parametrize("dtype,d,group", [(torch.bfloat16, 128, 4), (torch.bfloat16, 64, 1),
                                           (torch.float32, 64, 1), (torch.float32, 128, 2)])
def test_step_ragged_batch(dtype, d, group):
    say(f"step_ragged_batch dtype={dtype} d={d} G={group}")
    fin = F.Finch(H.finch_dtype(torch.empty(0, dtype=dtype)), d, group)
    specs = RAGGED_SPECS if dtype == torch.bfloat16 else [
        dict(s, n_que=min(s["n_que"], 24)) for s in RAGGED_SPECS]
    batch, ts = H.single_step_case(fin, specs, dtype, d, group, seed=100 + d + group)
    fin.step(batch)
    st = H.validate_single_step(ts, f"step {dtype} d={d}")
    say(f"  worst score rel err {st['worst_rel']:.2e}, near-tie swaps {st['swaps']}")
    fin.close()


def _which_scoring_kernels(fin, batch):
    F.finch_profile(fin.ctx, True)
    fin.step(batch)
    torch.cuda.synchronize()
    prof = F.finch_profile_read(fin.ctx)
    F.finch_profile(fin.ctx, False)
    return {k for k, v in prof.items() if v["launches"]}


PATHS = {"separate": F.FINCH_PATH_SEPARATE, "owner": F.FINCH_PATH_OWNER}


@pytest.mark.parametrize("d,group,path", [(128, 4, "separate"), (64, 8, "separate"), (128, 4, "owner"),
                                          (64, 2, "owner"), (128, 1, "owner"), (64, 8, "owner")])
def test_both_step_paths(d, group, path):
    """One kernel per stage and one workgroup per problem, each forced, on the same
    ragged batch."""
    say(f"both_step_paths d={d} G={group} {path}")
    fin = F.Finch(F.FINCH_BF16, d, group)
    fin.set_step_path(PATHS[path])
    cap = 512 // group
    specs = [dict(s, n_que=min(s["n_que"], cap)) for s in RAGGED_SPECS]
    specs += [dict(n_que=cap, c=1364, m=4096, r=1408), dict(n_que=max(1, cap // 3), c=5, m=130, r=64),
              dict(n_que=2, c=100, m=9000, r=900)]   # more candidates than a workgroup's registers hold
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, d, group, seed=300 + d + group)
    fin.step(batch)
    st = H.validate_single_step(ts, f"{path} d={d} G={group}")
    say(f"  worst score rel err {st['worst_rel']:.2e}, near-tie swaps {st['swaps']}")
    ran = _which_scoring_kernels(fin, batch)
    assert ran == {"owner": {"owner"}, "separate": {"rowstats", "colsum", "select", "gather"}}[path], ran
    # a second launch on the same context
    for t in ts:
        t["scores"].fill_(-5.0)
    fin.step(batch)
    H.validate_single_step(ts, f"{path} again")
    fin.close()


FP32_SPECS = [dict(n_que=16, c=48, m=256, r=64), dict(n_que=4, c=0, m=64, r=8), dict(n_que=1, c=7, m=0, r=3),
              dict(n_que=33, c=100, m=1300, r=333), dict(n_que=5, c=10, m=20, r=40), dict(n_que=9, c=0, m=700, r=0)]


@pytest.mark.parametrize("d,group", [(64, 1), (128, 2), (64, 5)])
def test_fp32_one_workgroup_per_problem(d, group):
    """fp32 inputs through the one-workgroup-per-problem kernels (vector ALU): the same
    results as the kernels per stage, to the oracle's tolerance."""
    say(f"fp32 owner d={d} G={group}")
    fin = F.Finch(F.FINCH_F32, d, group)
    fin.set_step_path(F.FINCH_PATH_OWNER)
    batch, ts = H.single_step_case(fin, FP32_SPECS, torch.float32, d, group, seed=70 + d)
    fin.step(batch)
    st = H.validate_single_step(ts, f"fp32 owner d={d} G={group}")
    say(f"  worst score rel err {st['worst_rel']:.2e}, near-tie swaps {st['swaps']}")
    assert _which_scoring_kernels(fin, batch) == {"owner"}
    fin.set_step_path(F.FINCH_PATH_SEPARATE)
    b2, t2 = H.single_step_case(fin, FP32_SPECS, torch.float32, d, group, seed=70 + d)
    fin.step(b2)
    H.validate_single_step(t2, f"fp32 per stage d={d} G={group}")
    fin.close()


def test_separate_entry_points_equal_step():
    """finch_score + finch_topk + finch_compact give what finch_step gives."""
    say("separate_entry_points")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    specs = [dict(n_que=48, c=300, m=1000, r=200), dict(n_que=12, c=0, m=700, r=64)]
    b1, t1 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=7)
    b2, t2 = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=7)
    fin.step(b1)
    fin.score(b2)
    fin.topk(b2)
    fin.compact(b2)
    torch.cuda.synchronize()
    for a, b in zip(t1, t2):
        for name in ("scores", "idx", "k_out", "v_out"):
            assert torch.equal(a[name], b[name]), name
    H.validate_single_step(t2, "separate")
    fin.close()


def test_step_with_scores_in_workspace():
    say("scores_in_workspace")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    specs = [dict(n_que=48, c=300, m=1000, r=200), dict(n_que=3, c=10, m=300, r=50)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=8, null_scores=True)
    fin.step(batch)
    H.validate_single_step(ts, "ws-scores", check_scores_too=False)
    fin.close()


@pytest.mark.parametrize("path", ["separate", "owner"])
def test_many_prompt_rows_are_chunked(path):
    """R = 4 * 160 = 640 rows: more than are staged at a time (512 with one kernel per
    stage, 256 with one workgroup per problem), so the keys are passed several times."""
    say(f"many_prompt_rows {path}")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(PATHS[path])
    specs = [dict(n_que=160, c=100, m=500, r=77), dict(n_que=130, c=0, m=300, r=20)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=9)
    fin.step(batch)
    st = H.validate_single_step(ts, "R=640")
    say(f"  worst score rel err {st['worst_rel']:.2e}")
    fin.close()


def test_many_slices_use_the_merge_kernel():
    """More than 16 key slices per problem: the slice statistics are merged by a
    kernel of their own instead of by pass 2."""
    say("many_slices")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_SLICE_KEYS, 256)
    specs = [dict(n_que=40, c=1000, m=4200, r=333), dict(n_que=3, c=0, m=290, r=20),
             dict(n_que=40, c=17, m=0, r=4)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=11)
    fin.step(batch)
    st = H.validate_single_step(ts, "20 slices")
    say(f"  worst score rel err {st['worst_rel']:.2e}")
    assert _which_scoring_kernels(fin, batch) == {"rowstats", "lse", "colsum", "select", "gather"}
    fin.close()


# A weight below 2^-126 cannot be held in fp32 (the kernels flush it to zero), so a score
# is only held to the stated tolerance while such weights cannot matter to it: above
# 1e-30 the flushed weights of all rows together stay below 1e-5 of the score.
FP32_UNDERFLOW_BOUND = 1e-30


def _check_above_underflow(got, want, what):
    """the stated per-element tolerance on every key whose score fp32 can hold; the others
    must be tiny too"""
    big = want > FP32_UNDERFLOW_BOUND
    rel = np.abs(got[big] - want[big]) / want[big]
    assert rel.max() <= H.SCORE_TOL["bf16"], f"{what}: rel err {rel.max():.3e} at key {np.nonzero(big)[0][rel.argmax()]}"
    assert (got[~big] <= 2 * FP32_UNDERFLOW_BOUND).all(), what


def test_large_logits_do_not_overflow():
    """Logits of several hundred: the running maximum keeps exp2 in range."""
    say("large_logits")
    fin = F.Finch(F.FINCH_BF16, 128, 1)
    specs = [dict(n_que=8, c=50, m=400, r=30, qscale=40.0)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 1, seed=10)
    fin.step(batch)
    torch.cuda.synchronize()
    got = ts[0]["scores"][:450].double().cpu().numpy()
    want = O.key_scores(W.to_numpy_storage(ts[0]["q"]), W.to_numpy_storage(ts[0]["k_cache"]),
                        W.to_numpy_storage(ts[0]["k_chunk"]))
    assert np.isfinite(got).all() and abs(got.sum() - 8.0) < 1e-3
    _check_above_underflow(got, want, "large logits")
    fin.close()


@pytest.mark.parametrize("path", ["separate", "owner"])
@pytest.mark.parametrize("kramp", [60.0, 1.0 / 60.0])
def test_logits_far_from_the_first_blocks_reference(kramp, path):
    """Key magnitudes rise (or fall) 60-fold along one slice, so the logits of later key
    blocks lie hundreds of powers of two above (below) those of the blocks a wave
    starts with: the reference of the running sums has to move (must not be needed)."""
    say(f"logit ramp x{kramp:.3g} {path}")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(PATHS[path])
    specs = [dict(n_que=12, c=0, m=3000, r=100, qscale=4.0, kramp=kramp),
             dict(n_que=40, c=10, m=2200, r=64, qscale=3.0, kramp=kramp)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=12)
    fin.step(batch)
    torch.cuda.synchronize()
    for t in ts:
        N, R = t["c"] + t["m"], 4 * t["n_que"]
        got = t["scores"][:N].double().cpu().numpy()
        want = O.key_scores(W.to_numpy_storage(t["q"]), W.to_numpy_storage(t["k_cache"]),
                            W.to_numpy_storage(t["k_chunk"]))
        assert np.isfinite(got).all() and abs(got.sum() - R) < 1e-3 * R
        _check_above_underflow(got, want, f"logit ramp x{kramp:.3g} {path}")
    fin.close()


def test_scores_sum_to_number_of_rows_and_are_reproducible():
    say("scores_sum / reproducible")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    specs = [dict(n_que=48, c=1364, m=4096, r=1408)]
    batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=11)
    fin.step(batch)
    torch.cuda.synchronize()
    s1, i1 = ts[0]["scores"].clone(), ts[0]["idx"].clone()
    assert abs(float(s1[:5460].double().sum()) - 192.0) < 1e-3
    for _ in range(3):
        ts[0]["scores"].fill_(-5.0)
        fin.step(batch)
        torch.cuda.synchronize()
        assert torch.equal(ts[0]["scores"], s1) and torch.equal(ts[0]["idx"], i1)
    fin.close()


# ------------------------------------------------------------------- top-r alone

def _topk_case(fin, score_arrays, rs):
    descs, keep = [], []
    for s, r in zip(score_arrays, rs):
        st = torch.from_numpy(np.asarray(s, dtype=np.float32)).cuda()
        n = st.numel()
        idx = torch.full((max(1, min(r, n)) + 1,), -9, dtype=torch.int32, device="cuda")
        descs.append(dict(q=None, k_cache=None, v_cache=None, k_chunk=None, v_chunk=None,
                          k_out=None, v_out=None, scores=st, idx=idx[:max(1, min(r, n))],
                          n_que=1, c=0, m=n, r=r))
        keep.append((st, idx))
    batch = F.Batch(descs)
    fin.topk(batch)
    torch.cuda.synchronize()
    for (st, idx), s, r in zip(keep, score_arrays, rs):
        want = O.top_r(np.asarray(s, dtype=np.float32), r)
        got = idx.cpu().numpy()
        assert np.array_equal(got[:len(want)], want), (r, len(s))
        assert got[max(1, len(want))] == -9


def test_topk_bit_exact_with_ties_and_signs():
    say("topk ties")
    fin = F.Finch(F.FINCH_BF16, 128, 1)
    rng = np.random.default_rng(21)
    cases, rs = [], []
    for n, r in [(5460, 1408), (5460, 1), (5460, 5459), (1025, 512), (1024, 1000), (63, 7),
                 (1, 1), (3000, 0), (20000, 7000), (70000, 33333)]:
        cases.append(rng.standard_normal(n).astype(np.float32)); rs.append(r)
        cases.append(rng.integers(0, 4, n).astype(np.float32) * 0.25); rs.append(r)   # 4 values
        cases.append(np.full(n, 0.125, np.float32)); rs.append(r)                     # all tied
    mixed = rng.integers(-3, 3, 4000).astype(np.float32)
    mixed[::7] = -0.0
    cases.append(mixed); rs.append(1700)
    tiny = (rng.random(3000) * 1e-38).astype(np.float32)          # denormals included
    cases.append(tiny); rs.append(900)
    _topk_case(fin, cases, rs)
    fin.close()


# --------------------------------------------------------------- chunk loops

def test_c1_full_workload():
    """C1 exactly as specified: every problem, every step, fp32 tolerance."""
    say("C1 full")
    w = W.get_workload("C1")
    fin = F.Finch(F.FINCH_F32, w.head_dim, w.group)
    probs = [H.make_gpu_problem(w, b, l, g) for b, l, g in W.problems_of(w)]
    loop = ChunkLoop(fin, probs, w.chunk, history=True)
    assert [r for r in loop.rs[0]] == [16, 32, 48, 64]
    F.finch_profile(fin.ctx, True)
    loop.run()
    torch.cuda.synchronize()
    prof = F.finch_profile_read(fin.ctx)
    F.finch_profile(fin.ctx, False)
    # the whole loop of the batch is one launch
    assert {k: v["launches"] for k, v in prof.items() if v["launches"]} == {"owner": 1}, prof
    st = H.validate_chunk_loop(loop, range(len(probs)), "C1")
    say(f"  C1: {st}")
    # ... and one kernel per stage, step by step, gives the same selection
    fin.set_step_path(F.FINCH_PATH_SEPARATE)
    loop2 = ChunkLoop(fin, probs, w.chunk, history=True)
    loop2.run()
    H.validate_chunk_loop(loop2, range(len(probs)), "C1 per stage")
    assert torch.equal(loop.idx, loop2.idx)
    fin.set_step_path(F.FINCH_PATH_AUTO)
    # the planted keys are what the method is supposed to keep
    for p, pb in enumerate(probs):
        Kt, _ = loop.final_cache(p)
        planted_rows = pb["K"][pb["planted"]]
        found = sum(bool((Kt == row).all(dim=1).any()) for row in planted_rows)
        assert found == 8
    fin.close()


@pytest.mark.parametrize("name,n_cont,problems", [
    ("C2", None, [(0, 0, 0), (0, 7, 13), (0, 31, 31)]),
    ("C3", 8192, [(0, 0, 0), (0, 5, 3)]),
    ("C4", 16384, [(0, 0, 0), (0, 9, 7)]),
    ("C5", None, None),
])
def test_workload_shaped_chunk_loops(name, n_cont, problems):
    """Each bf16 workload's geometry, recipe and schedule on a few problems (C3/C4
    with a shortened document so the oracle finishes in seconds); C5: the three
    shortest requests, one KV head each, full ragged length mix."""
    say(f"{name} shaped chunk loop")
    w = W.get_workload(name)
    fin = F.Finch(F.FINCH_BF16, w.head_dim, w.group)
    if name == "C5":
        order = sorted(range(len(w.requests)), key=lambda b: w.requests[b].n_cont)[:3]
        problems = [(b, b % w.layers, b % w.kv_heads) for b in order]
    probs = []
    for b, l, g in problems:
        pb = H.make_gpu_problem(w, b, l, g, n_cont=n_cont)
        if n_cont is not None:
            pb["budget"] = max(1, n_cont * w.requests[b].budget // w.requests[b].n_cont)
        probs.append(pb)
    loop = ChunkLoop(fin, probs, w.chunk, history=True)
    loop.run()
    st = H.validate_chunk_loop(loop, range(len(probs)), name)
    say(f"  {name}: {st}")
    fin.close()


def test_per_step_queries_and_resume():
    """A different Q at every step, and split-and-resume == straight run."""
    say("per-step Q / resume")
    w = W.get_workload("C2")
    fin = F.Finch(F.FINCH_BF16, 128, 1)
    pb = H.make_gpu_problem(w, 0, 1, 2, n_cont=2048)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    pb["Q"] = [H.rand_storage((32, 128), torch.bfloat16, gen) for _ in range(4)]
    pb["budget"] = 512
    loop = ChunkLoop(fin, [pb], 512, history=True)
    loop.run()
    H.validate_chunk_loop(loop, [0], "per-step Q")
    Kt, Vt = (t.clone() for t in loop.final_cache(0))
    # resume: first two steps, then continue by hand from the saved cache
    half = dict(pb, K=pb["K"][:1024], V=pb["V"][:1024], Q=pb["Q"][:2], budget=256)
    l2 = ChunkLoop(fin, [half], 512, history=True)
    l2.run()
    torch.cuda.synchronize()
    assert l2.rs[0] == loop.rs[0][:2]
    Kc, Vc = (t.clone() for t in l2.final_cache(0))
    for i in (2, 3):
        r = loop.rs[0][i]
        t = dict(q=pb["Q"][i], k_cache=Kc, v_cache=Vc, k_chunk=pb["K"][512 * i:512 * i + 512],
                 v_chunk=pb["V"][512 * i:512 * i + 512],
                 k_out=torch.empty(r, 128, dtype=torch.bfloat16, device="cuda"),
                 v_out=torch.empty(r, 128, dtype=torch.bfloat16, device="cuda"),
                 scores=torch.empty(Kc.shape[0] + 512, device="cuda"),
                 idx=torch.empty(r, dtype=torch.int32, device="cuda"),
                 n_que=32, c=Kc.shape[0], m=512, r=r)
        fin.step(F.Batch([t]))
        torch.cuda.synchronize()
        Kc, Vc = t["k_out"], t["v_out"]
    assert torch.equal(Kc, Kt) and torch.equal(Vc, Vt)
    fin.close()


@pytest.mark.parametrize("path", ["owner", "separate"])
def test_whole_loop_call_equals_step_by_step(path):
    """finch_loop (one launch for all steps with one workgroup per slot, or its
    step-by-step form) against one finch_step per chunk: problems of different
    lengths (slots drop out from the end), a different Q per step for some, and the
    oracle on every step of every problem."""
    say(f"whole loop vs step by step ({path})")
    w = W.get_workload("C4")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(PATHS[path])
    gen = torch.Generator(device="cuda"); gen.manual_seed(21)
    lengths = [1500, 4096, 2600, 520, 3333, 4096]
    probs = []
    for j, n in enumerate(lengths):
        pb = H.make_gpu_problem(w, 0, 0, j, n_cont=n)
        pb["budget"] = max(8, n // 7)
        if j % 2:
            steps = (n + 511) // 512
            pb["Q"] = [H.rand_storage(tuple(pb["Q"].shape), torch.bfloat16, gen) for _ in range(steps)]
        probs.append(pb)
    loops = []
    for per_step in (False, True):
        loop = ChunkLoop(fin, probs, 512, history=True)
        loop.run(per_step=per_step)
        st = H.validate_chunk_loop(loop, list(range(len(probs))), f"loop per_step={per_step}")
        say(f"  per_step={per_step}: {st}")
        loops.append(loop)
    a, b = loops
    assert torch.equal(a.scores, b.scores) and torch.equal(a.idx, b.idx)
    for p in range(len(probs)):
        for x, y in zip(a.final_cache(p), b.final_cache(p)):
            assert torch.equal(x, y)
    fin.close()


def test_loop_step_table_is_checked():
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    batch, ts = H.single_step_case(fin, [dict(n_que=4, c=0, m=64, r=8)] * 3, torch.bfloat16, 128, 4, seed=3)
    fin.reserve(batch)
    dev_first = torch.tensor([0, 2, 3], dtype=torch.int32, device="cuda")

    def call(first):
        arr = (ctypes.c_int32 * len(first))(*first)
        F.finch_loop(fin.ctx, batch.host, batch.dev_ptr, arr, dev_first.data_ptr(), len(first) - 1,
                     fin.ws.data_ptr(), fin.ws.numel(), 0)

    for bad in ([0, 1, 3], [1, 2, 3], [0, 2, 1]):   # growing step, not starting at 0, negative count
        with pytest.raises(F.FinchError) as e:
            call(bad)
        assert e.value.status == F.FINCH_ERR_INVALID_ARG
    call([0, 2, 3])
    torch.cuda.synchronize()
    fin.close()


# --------------------------------------------------------------- error handling

def test_argument_errors_are_reported_before_any_launch():
    say("argument errors")
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    batch, ts = H.single_step_case(fin, [dict(n_que=4, c=10, m=100, r=20)], torch.bfloat16, 128, 4, 3)
    need = fin.reserve(batch)
    lib = F.load_library()
    ws, stream = fin.ws.data_ptr(), torch.cuda.current_stream().cuda_stream

    def call(name, host, n=1, ws_ptr=ws, ws_bytes=None, dev=batch.dev_ptr):
        return getattr(lib, name)(fin.ctx, host, ctypes.c_void_p(dev), n, ctypes.c_void_p(ws_ptr),
                                  need if ws_bytes is None else ws_bytes, ctypes.c_void_p(stream))

    def variant(**kw):
        h = (F.finch_problem * 1)()
        ctypes.memmove(h, batch.host, ctypes.sizeof(F.finch_problem))
        for k, v in kw.items():
            setattr(h[0], k, v)
        return h

    assert call("finch_step", batch.host) == F.FINCH_OK
    assert call("finch_step", variant(q=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(q=ts[0]["q"].data_ptr() + 2)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(k_chunk=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(v_cache=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(idx=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(n_que=0)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(c=-1)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(r=-5)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(k_out=ts[0]["k_chunk"].data_ptr())) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(v_out=ts[0]["v_cache"].data_ptr() + 256)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", variant(v_out=ts[0]["k_out"].data_ptr())) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_score", variant(scores=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_topk", variant(scores=None)) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", batch.host, ws_bytes=need - 1) == F.FINCH_ERR_WORKSPACE
    assert call("finch_step", batch.host, ws_ptr=ws + 8) == F.FINCH_ERR_WORKSPACE
    assert call("finch_step", batch.host, ws_ptr=0) == F.FINCH_ERR_WORKSPACE
    assert call("finch_step", batch.host, n=-1) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", batch.host, dev=0) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", None) == F.FINCH_ERR_INVALID_ARG
    assert call("finch_step", batch.host, n=0) == F.FINCH_OK
    assert call("finch_step", variant(c=1 << 25)) == F.FINCH_ERR_CAPACITY
    torch.cuda.synchronize()
    H.validate_single_step(ts, "after error calls")
    fin.close()
