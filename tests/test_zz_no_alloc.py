"""finch_step_static (the step on the library's own scratch array: for callers that
cannot allocate) against finch_step, through the C ABI: two calls in a row, the second
with a smaller input, bit for bit and against the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2408_00167_amd as F
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

BIG = [dict(n_que=48, c=700, m=2100, r=650), dict(n_que=48, c=0, m=2500, r=300),
       dict(n_que=17, c=333, m=1000, r=1), dict(n_que=48, c=1364, m=4096, r=1408)]
SMALL = [dict(n_que=5, c=40, m=130, r=60), dict(n_que=48, c=0, m=77, r=200)]


def _outputs(ts):
    torch.cuda.synchronize()
    out = []
    for t in ts:
        out.append((None if t["scores"] is None else t["scores"].clone(), t["idx"].clone(),
                    t["k_out"].clone(), t["v_out"].clone()))
    return out


def _same(a, b, what):
    for n, (x, y) in enumerate(zip(a, b)):
        for u, v, name in zip(x, y, ("scores", "idx", "k_out", "v_out")):
            if u is None:
                assert v is None
                continue
            assert torch.equal(u.view(torch.uint8) if u.dtype != torch.int32 else u,
                               v.view(torch.uint8) if v.dtype != torch.int32 else v), f"{what} problem {n}: {name}"


@pytest.mark.parametrize("path", [F.FINCH_PATH_SEPARATE, F.FINCH_PATH_AUTO])
@pytest.mark.parametrize("null_scores", [False, True])
def test_step_static_matches_step(path, null_scores):
    lib = F.load_library()
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(path)
    stream = torch.cuda.current_stream().cuda_stream
    for call, specs in enumerate((BIG, SMALL)):
        # the same seeded inputs twice: once through finch_step with a workspace, once
        # through finch_step_static
        ref_batch, ref_ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=40 + call,
                                               null_scores=null_scores)
        fin.step(ref_batch)
        want = _outputs(ref_ts)
        batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=40 + call,
                                       null_scores=null_scores)
        need = F.finch_workspace_size(fin.ctx, batch.host, batch.n)
        assert 0 < need <= F.finch_static_scratch_bytes()
        st = lib.finch_step_static(fin.ctx, batch.host, ctypes.c_void_p(batch.dev_ptr), batch.n,
                                   ctypes.c_void_p(stream))
        assert st == F.FINCH_OK, st
        _same(_outputs(ts), want, f"call {call}")
        H.validate_single_step(ts, f"step_static call {call}")
    fin.close()


def test_step_static_fp32_and_layer_group():
    fin = F.Finch(F.FINCH_F32, 64, 1)
    for call, specs in enumerate(([dict(n_que=16, c=48, m=256, r=64)] * 4, [dict(n_que=3, c=0, m=50, r=20)])):
        ref_batch, ref_ts = H.single_step_case(fin, specs, torch.float32, 64, 1, seed=50 + call)
        fin.step(ref_batch)
        want = _outputs(ref_ts)
        batch, ts = H.single_step_case(fin, specs, torch.float32, 64, 1, seed=50 + call)
        fin.step_static(batch)
        _same(_outputs(ts), want, f"fp32 call {call}")
        H.validate_single_step(ts, f"step_static fp32 call {call}")
    fin.close()
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    F.finch_set_option(fin.ctx, F.FINCH_OPT_LAYER_GROUP, 2)
    for call, specs in enumerate(([dict(n_que=48, c=300, m=900, r=200)] * 4, [dict(n_que=8, c=10, m=100, r=30)] * 2)):
        ref_batch, ref_ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=60 + call)
        fin.step(ref_batch)
        want = _outputs(ref_ts)
        batch, ts = H.single_step_case(fin, specs, torch.bfloat16, 128, 4, seed=60 + call)
        fin.step_static(batch)
        _same(_outputs(ts), want, f"layer call {call}")
    fin.close()


def test_step_static_refuses_what_does_not_fit():
    lib = F.load_library()
    fin = F.Finch(F.FINCH_BF16, 128, 4)
    fin.set_step_path(F.FINCH_PATH_SEPARATE)
    # descriptors are only sized on the host here: nothing is launched for a refused batch
    specs = [dict(n_que=48, c=1364, m=4096, r=1408)] * 1024
    hd = (F.finch_problem * len(specs))()
    for d, sp in zip(hd, specs):
        d.n_que, d.c, d.m, d.r = sp["n_que"], sp["c"], sp["m"], sp["r"]
    need = F.finch_workspace_size(fin.ctx, hd, len(specs))
    assert need > F.finch_static_scratch_bytes()
    dummy = torch.zeros(len(specs) * ctypes.sizeof(F.finch_problem), dtype=torch.uint8, device="cuda")
    st = lib.finch_step_static(fin.ctx, hd, ctypes.c_void_p(dummy.data_ptr()), len(specs), None)
    assert st == F.FINCH_ERR_CAPACITY
    fin.close()
