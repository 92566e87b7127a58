"""Host-side checks of bench.py that need no GPU: more than one GPU is refused with a
message, and the byte / flop accounting matches hand-computed values on a tiny loop."""
import os
import subprocess
import sys
import types

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and "--gpus 1" in r.stderr
    assert not r.stdout.strip().startswith("{")


def test_byte_and_flop_accounting():
    sys.path.insert(0, ROOT)
    import bench
    # two problems, two steps; shapes (c, m, r) per active problem
    w = types.SimpleNamespace(elem_bytes=2, head_dim=128, group=4)
    loop = types.SimpleNamespace(
        n_steps=2, active=[[0, 1], [0]],
        step_shapes=[[(0, 100, 10), (0, 50, 50)], [(10, 100, 20)]],
        problems=[dict(n_que=3), dict(n_que=5)])
    per, total, keys = bench.algorithmic_bytes(w, loop)
    row = 128 * 2
    assert keys == 100 + 50 + 110
    # every key once + the prompt rows once per step, per problem
    assert per["score_pass"] == (100 + 12) * row + (50 + 20) * row + (110 + 12) * row
    # kept rows of K and V read once and written once
    assert per["gather"] == (10 + 50 + 20) * row * 4
    assert total == per["score_pass"] + per["gather"]
    assert bench.logit_flops(w, loop) == 2 * 2 * 128 * (100 * 12 + 50 * 20 + 110 * 12)
