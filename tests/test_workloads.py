"""The seeded input recipes: shapes, determinism, and the structure each recipe
promises (planted keys, channel outliers, rotation keeps norms).  CPU only."""
import math

import numpy as np
import torch

import workloads as W


def test_shapes_and_counts():
    c1, c2, c3, c4, c5 = (W.get_workload(n) for n in ("C1", "C2", "C3", "C4", "C5"))
    assert (c1.n_problems, c2.n_problems, c3.n_problems, c4.n_problems, c5.n_problems) == \
        (4, 1024, 256, 256, 4096)
    assert [w.rows(w.requests[0]) for w in (c1, c2, c3, c4)] == [16, 32, 256, 192]
    assert c4.n_planted(c4.requests[0]) == 655 and c2.n_planted(c2.requests[0]) == 41
    assert len(c5.requests) == 16
    for r in c5.requests:
        assert 2048 <= r.n_cont <= 65536 and 16 <= r.n_que <= 128 and r.budget == r.n_cont // 32
    assert len(list(W.problems_of(c4))) == 256


def test_deterministic_and_independent():
    w = W.get_workload("C1")
    a = W.make_problem(w, 0, 0, 2)
    b = W.make_problem(w, 0, 0, 2)
    c = W.make_problem(w, 0, 0, 3)
    for key in ("Q", "K", "V"):
        assert torch.equal(a[key], b[key])
        assert not torch.equal(a[key], c[key])
    assert a["Q"].shape == (16, 64) and a["K"].shape == (1024, 64) and a["K"].dtype == torch.float32
    assert len({W.problem_seed(w, 0, 0, g) for g in range(4)}) == 4


def test_c1_planted_keys_are_three_times_mean_query():
    w = W.get_workload("C1")
    p = W.make_problem(w, 0, 0, 1)
    qbar = p["Q"].mean(dim=0)
    assert p["planted"].numel() == 8
    assert torch.allclose(p["K"][p["planted"]], (3.0 * qbar).expand(8, -1))


def test_c2_rotation_and_alignment():
    w = W.get_workload("C2")
    p = W.make_problem(w, 0, 3, 5, n_cont=512)
    assert p["K"].dtype == torch.bfloat16 and p["K"].shape == (512, 128)
    k = p["K"].float()
    norms = k.norm(dim=1)
    mask = torch.ones(512, dtype=torch.bool)
    mask[p["planted"]] = False
    assert abs(float(norms[mask].mean()) - math.sqrt(128)) < 0.5      # rotation keeps norms
    qbar = p["Q"].float().mean(dim=0)
    cos = torch.nn.functional.cosine_similarity(k[p["planted"]], qbar[None, :], dim=1)
    assert (cos > 0.99).all()


def test_c3_outlier_channels():
    w = W.get_workload("C3")
    p = W.make_problem(w, 0, 1, 2, n_cont=4096)
    std = p["K"].float().std(dim=0)
    assert int(((std < 0.9) | (std > 1.1)).sum()) <= 4
    assert int(((std > 0.9) & (std < 1.1)).sum()) >= 124


def test_storage_round_trip():
    t = torch.randn(5, 8).to(torch.bfloat16)
    a = W.to_numpy_storage(t)
    assert a.dtype == np.uint16
    assert torch.equal(W.from_numpy_storage(a), t)
    f = torch.randn(3, 4)
    assert torch.equal(W.from_numpy_storage(W.to_numpy_storage(f)), f)
