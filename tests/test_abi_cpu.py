"""Host-side checks of the C-ABI library that need no GPU: it loads, it exports
every function include/finch.h declares, and its host-only entry points behave."""
import ctypes
import os
import re

import pytest
import torch

import paper_2408_00167_amd as F
from oracle import finch_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    with open(os.path.join(ROOT, "include", "finch.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(finch_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    lib = F.load_library()
    names = declared_functions()
    assert set(names) == set(F.EXPORTED_SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None
    assert F.finch_version() >= 100


def test_problem_struct_layout_matches_header():
    assert ctypes.sizeof(F.finch_problem) == 112
    assert F.finch_problem.n_que.offset == 72 and F.finch_problem.r.offset == 84
    assert ctypes.sizeof(F.finch_config) == 16


def test_schedule_matches_paper_rule_and_oracle():
    assert F.finch_schedule(1024, 256, 64) == [16, 32, 48, 64]
    assert F.finch_schedule(131072, 4096, 1408) == [44 * i for i in range(1, 33)]
    for n_cont, m, k in [(1000, 256, 100), (2049, 2048, 64), (5, 8, 2), (4096, 512, 5000),
                         (777, 100, 777), (65536, 2048, 2048), (3000, 7, 1), (40000, 2048, 1250),
                         (1 << 33, 1 << 20, 12345)]:
        assert F.finch_schedule(n_cont, m, k) == O.schedule(n_cont, m, k)
        assert F.finch_schedule(n_cont, m, k, constant_budget=True) == O.schedule(n_cont, m, k, constant_budget=True)
    assert F.finch_schedule(0, 16, 4) == []


def test_schedule_argument_errors():
    lib = F.load_library()
    buf = (ctypes.c_int32 * 4)()
    assert lib.finch_schedule(100, 0, 10, buf, 4) == F.FINCH_ERR_INVALID_ARG
    assert lib.finch_schedule(-1, 8, 10, buf, 4) == F.FINCH_ERR_INVALID_ARG
    assert lib.finch_schedule(100, 8, 10, buf, 4) == F.FINCH_ERR_CAPACITY      # needs 13 slots
    assert lib.finch_schedule(100, 50, 10, None, 4) == F.FINCH_ERR_INVALID_ARG
    assert lib.finch_status_string(F.FINCH_ERR_WORKSPACE).decode().startswith("workspace")


def test_create_rejects_bad_configs_before_touching_the_gpu():
    lib = F.load_library()
    ctx = ctypes.c_void_p()
    for cfg, want in [(F.finch_config(2, 128, 1, 0), F.FINCH_ERR_UNSUPPORTED),
                      (F.finch_config(F.FINCH_BF16, 96, 1, 0), F.FINCH_ERR_UNSUPPORTED),
                      (F.finch_config(F.FINCH_BF16, 128, 0, 0), F.FINCH_ERR_UNSUPPORTED),
                      (F.finch_config(F.FINCH_BF16, 128, 4, 7), F.FINCH_ERR_INVALID_ARG)]:
        assert lib.finch_create(ctypes.byref(cfg), ctypes.byref(ctx)) == want
        assert not ctx.value
    assert lib.finch_create(None, ctypes.byref(ctx)) == F.FINCH_ERR_INVALID_ARG


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful without a GPU")
def test_no_gpu_means_loud_failure_not_fallback():
    with pytest.raises(RuntimeError):
        F.Finch(F.FINCH_BF16, 128, 4)
    with pytest.raises(F.FinchError) as e:
        F.finch_create(F.FINCH_BF16, 128, 4)
    assert e.value.status == F.FINCH_ERR_HIP


def _loop_descs(n_slots, n_steps, d=128, c_step=8, m=64, overlap=None):
    """Descriptors of a chunk loop laid out by hand in a made-up address space (the
    library only compares the pointers): per slot a document K and V, two ping-pong
    cache slabs, idx and scores per step.  `overlap` plants one violation."""
    rb = d * 2
    cap = c_step * n_steps
    slot_bytes = 2 * (m * n_steps) * rb + 4 * cap * rb + n_steps * (cap * 4 + (cap + m) * 4) + 4096
    slot_bytes = (slot_bytes + 255) // 256 * 256
    base0 = 1 << 32
    hd = (F.finch_problem * (n_slots * n_steps))()
    first = (ctypes.c_int32 * (n_steps + 1))(*[s * n_slots for s in range(n_steps + 1)])
    qaddr = base0 - (1 << 20)
    for s in range(n_steps):
        for j in range(n_slots):
            b = base0 + j * slot_bytes
            kdoc, vdoc = b, b + m * n_steps * rb
            slabs = vdoc + m * n_steps * rb
            kslab = [slabs, slabs + cap * rb]
            vslab = [slabs + 2 * cap * rb, slabs + 3 * cap * rb]
            misc = slabs + 4 * cap * rb
            pd = hd[s * n_slots + j]
            pd.q = qaddr                      # one prompt block read by every slot
            pd.n_que, pd.c, pd.m, pd.r = 4, c_step * s, m, c_step * (s + 1)
            pd.k_cache, pd.v_cache = (kslab[s % 2], vslab[s % 2]) if s else (None, None)
            pd.k_chunk, pd.v_chunk = kdoc + s * m * rb, vdoc + s * m * rb
            pd.k_out, pd.v_out = kslab[(s + 1) % 2], vslab[(s + 1) % 2]
            pd.idx = misc + s * (cap * 4 + (cap + m) * 4)
            pd.scores = pd.idx + cap * 4
    if overlap == "write_into_other_slots_chunk":
        hd[1 * n_slots + 0].k_out = hd[2 * n_slots + 1].k_chunk      # slot 0 writes keys slot 1 reads later
    elif overlap == "shared_idx":
        hd[0 * n_slots + 2].idx = hd[1 * n_slots + 3].idx            # two slots write one index array
    elif overlap == "partial":
        hd[2 * n_slots + 1].v_out = hd[2 * n_slots + 2].v_cache + rb * 3
    return hd, first


def test_loop_check_accepts_disjoint_slots_and_rejects_overlaps_between_slots():
    n_slots, n_steps = 5, 4
    hd, first = _loop_descs(n_slots, n_steps)
    assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, first, n_steps) == F.FINCH_OK
    for bad in ("write_into_other_slots_chunk", "shared_idx", "partial"):
        hd, first = _loop_descs(n_slots, n_steps, overlap=bad)
        assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, first, n_steps) == F.FINCH_ERR_INVALID_ARG, bad
    # a slot may read what it wrote itself in an earlier step (that is the chunk loop),
    # and one slot alone has nobody to collide with
    hd, first = _loop_descs(1, n_steps)
    assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, first, n_steps) == F.FINCH_OK
    # the other checks of finch_loop are made too: a step table that grows, an output on its source
    hd, first = _loop_descs(n_slots, n_steps)
    grow = (ctypes.c_int32 * (n_steps + 1))(0, 2, 7, 12, 20)
    assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, grow, n_steps) == F.FINCH_ERR_INVALID_ARG
    hd[n_slots].k_out = hd[n_slots].k_chunk
    assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, first, n_steps) == F.FINCH_ERR_INVALID_ARG
    assert F.finch_loop_check(F.FINCH_BF16, 96, 1, hd, first, n_steps) == F.FINCH_ERR_UNSUPPORTED


def test_loop_check_many_slots_is_fast():
    import time
    hd, first = _loop_descs(1024, 8)
    t0 = time.perf_counter()
    assert F.finch_loop_check(F.FINCH_BF16, 128, 1, hd, first, 8) == F.FINCH_OK
    assert time.perf_counter() - t0 < 0.5
