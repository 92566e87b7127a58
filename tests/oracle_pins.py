"""Pins for the CPU oracle, written as functions of the oracle module `O` so that
the same checks can be run against deliberately broken copies of it
(test_oracle_mutations.py).  Expected values here come from closed forms worked
out by hand, from library routines (scipy, numpy argsort), from pure-Python brute
force, or from the paper (tests/golden/); none come from the oracle itself.
"""
import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (round to nearest even), test helper."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


# ----------------------------------------------------------------- closed forms

def pin_onehot_closed_form(O):
    # d = 4 so sqrt(d_k) = 2.  Row 0 has logits (2, 0, 0), row 1 has (0, 4, 0).
    Q = np.array([[2, 0, 0, 0], [0, 4, 0, 0]], dtype=np.float32)
    K = np.array([[2, 0, 0, 0], [0, 2, 0, 0], [0, 0, 2, 0]], dtype=np.float32)
    e2, e4 = math.exp(2.0), math.exp(4.0)
    want = np.array([[e2 / (e2 + 2), 1 / (e2 + 2), 1 / (e2 + 2)],
                     [1 / (e4 + 2), e4 / (e4 + 2), 1 / (e4 + 2)]])
    P = O.attention_weights(Q, K)
    assert P.shape == (2, 3)
    np.testing.assert_allclose(P, want, rtol=1e-14, atol=0)
    s = O.key_scores(Q, K[:1], K[1:])
    np.testing.assert_allclose(s, want.sum(axis=0), rtol=1e-14, atol=0)
    # the best key overall is key 1 (e4-dominated), then key 0
    assert list(O.top_r(s, 1)) == [1]
    assert list(O.top_r(s, 2)) == [0, 1]


def pin_two_key_sigmoid(O):
    # one query, two keys: the weight of key 0 is the logistic function of the
    # logit difference (q.k0 - q.k1)/sqrt(d).
    q = np.array([[1.0, 2.0, -1.0, 0.5, 0, 0, 0, 0, 0]], dtype=np.float64)  # d = 9 -> sqrt = 3
    k0 = np.array([3.0, 0, 0, 0, 0, 0, 0, 0, 0])
    k1 = np.array([0, 0, 3.0, 0, 0, 0, 0, 0, 0])
    delta = (3.0 * 1.0 - 3.0 * (-1.0)) / 3.0        # = 2
    s = O.key_scores(q, np.stack([k0]), np.stack([k1]))
    np.testing.assert_allclose(s, [1 / (1 + math.exp(-delta)), 1 / (1 + math.exp(delta))],
                               rtol=1e-14)


def pin_identical_keys_uniform(O):
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((7, 16)).astype(np.float32)
    key = rng.standard_normal(16).astype(np.float32)
    K = np.tile(key, (10, 1))
    s = O.key_scores(Q, K[:4], K[4:])
    np.testing.assert_allclose(s, np.full(10, 7 / 10), rtol=1e-13)
    # exact ties everywhere -> the lowest indices win
    assert list(O.top_r(np.full(10, 0.7), 4)) == [0, 1, 2, 3]


def pin_dominant_key(O):
    # one key far above the rest takes (almost) all of every row: score -> R
    rng = np.random.default_rng(6)
    Q = np.abs(rng.standard_normal((5, 8))) + 0.5
    K = rng.standard_normal((12, 8)) * 0.01
    K[9] = 50.0                     # logit >= 50*8*0.5/sqrt(8) for every row
    s = O.key_scores(Q, K[:3], K[3:])
    assert abs(s[9] - 5.0) < 1e-9 and s.argmax() == 9


def pin_single_row_is_argsort_of_dots(O):
    rng = np.random.default_rng(7)
    q = rng.standard_normal((1, 32))
    K = rng.standard_normal((200, 32))
    dots = K @ q[0]
    want = np.sort(np.argsort(-dots, kind="stable")[:37])
    got = O.top_r(O.key_scores(q, K[:50], K[50:]), 37)
    assert got.dtype == np.int32 and list(got) == list(want)


def pin_scipy_softmax(O):
    from scipy.special import logsumexp, softmax
    rng = np.random.default_rng(8)
    Q = rng.standard_normal((9, 24)) * 2
    K = rng.standard_normal((41, 24)) * 2
    S = np.einsum("id,jd->ij", Q, K) / math.sqrt(24)
    P = O.attention_weights(Q, K)
    np.testing.assert_allclose(P, softmax(S, axis=1), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(O.key_scores(Q, K[:11], K[11:]),
                               np.exp(S - logsumexp(S, axis=1, keepdims=True)).sum(axis=0),
                               rtol=1e-12)


# ------------------------------------------------------------------ brute force

def brute_scores(Q, Kc, Kk):
    """Explicit full softmax matrix in pure Python floats, then column sums."""
    keys = [list(map(float, row)) for row in Kc] + [list(map(float, row)) for row in Kk]
    d = len(Q[0])
    out = [0.0] * len(keys)
    for qrow in Q:
        logits = [sum(float(a) * b for a, b in zip(qrow, k)) / math.sqrt(d) for k in keys]
        top = max(logits)
        ex = [math.exp(x - top) for x in logits]
        z = math.fsum(ex)
        for j, e in enumerate(ex):
            out[j] += e / z
    return out


def brute_top(scores, r):
    order = sorted(range(len(scores)), key=lambda j: (-scores[j], j))
    return sorted(order[:max(0, min(r, len(scores)))])


def pin_brute_force_tiny(O):
    rng = np.random.default_rng(9)
    for (R, c, m, d, r) in [(1, 0, 5, 4, 2), (3, 4, 6, 8, 5), (4, 7, 0, 8, 3),
                            (6, 5, 9, 16, 14), (2, 3, 3, 2, 0), (5, 2, 11, 4, 20)]:
        Q = rng.standard_normal((R, d)).astype(np.float32)
        Kc = rng.standard_normal((c, d)).astype(np.float32)
        Kk = rng.standard_normal((m, d)).astype(np.float32)
        Vc = rng.standard_normal((c, d)).astype(np.float32)
        Vk = rng.standard_normal((m, d)).astype(np.float32)
        want = brute_scores(Q, Kc, Kk)
        scores, idx, Kn, Vn = O.step(Q, Kc, Vc, Kk, Vk, r)
        np.testing.assert_allclose(scores, want, rtol=1e-12)
        widx = brute_top(want, r)
        assert list(idx) == widx
        allK = [row for row in Kc] + [row for row in Kk]
        allV = [row for row in Vc] + [row for row in Vk]
        assert Kn.shape == (len(widx), d) and Vn.shape == (len(widx), d)
        for t, j in enumerate(widx):
            assert Kn[t].tobytes() == allK[j].tobytes()
            assert Vn[t].tobytes() == allV[j].tobytes()


def pin_brute_force_bf16(O):
    rng = np.random.default_rng(10)
    Qf = rng.standard_normal((3, 8)).astype(np.float32)
    Kf = rng.standard_normal((9, 8)).astype(np.float32)
    Qb, Kb = bf16_bits(Qf), bf16_bits(Kf)
    # widen by hand: bf16 bits are the top half of a float32
    def wide(bits):
        return (bits.astype(np.uint32) << 16).view(np.float32)
    want = brute_scores(wide(Qb), wide(Kb[:4]), wide(Kb[4:]))
    got = O.key_scores(Qb, Kb[:4], Kb[4:])
    np.testing.assert_allclose(got, want, rtol=1e-12)
    # gather keeps the uint16 bits
    g = O.gather_rows(np.array([1, 8]), Kb[:4], Kb[4:])
    assert g.dtype == np.uint16 and g.tobytes() == Kb[[1, 8]].tobytes()


def pin_widen_bits(O):
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x8000, 0x4049], dtype=np.uint16)
    want = [1.0, -2.0, 1.5, 0.0, -0.0, 3.140625]
    got = O.widen(bits)
    assert got.dtype == np.float64 and list(got) == want
    assert math.copysign(1.0, got[4]) == -1.0
    x32 = np.array([0.1, -7.25], dtype=np.float32)
    assert list(O.widen(x32)) == [float(x32[0]), -7.25]


# ------------------------------------------------------------------- invariants

def pin_invariants(O):
    rng = np.random.default_rng(11)
    for trial in range(6):
        R, c, m, d = rng.integers(1, 12), rng.integers(0, 30), rng.integers(1, 40), 16
        Q = rng.standard_normal((R, d)).astype(np.float32) * 3
        Kc = rng.standard_normal((c, d)).astype(np.float32)
        Kk = rng.standard_normal((m, d)).astype(np.float32)
        K = np.concatenate([Kc, Kk])
        P = O.attention_weights(Q, K)
        np.testing.assert_allclose(P.sum(axis=1), np.ones(R), rtol=1e-13)
        assert (P > 0).all()
        s = O.key_scores(Q, Kc, Kk)
        assert abs(s.sum() - R) < 1e-11 * R
        N = c + m
        for r in (0, 1, N // 2, N, N + 5):
            idx = O.top_r(s, r)
            assert len(idx) == min(r, N)
            assert (np.diff(idx) > 0).all()
            kept = np.zeros(N, bool)
            kept[idx] = True
            if 0 < len(idx) < N:
                assert s[kept].min() >= s[~kept].max()
            if r >= N:
                assert list(idx) == list(range(N))
        # permuting keys permutes scores
        perm = rng.permutation(N)
        s_perm = O.key_scores(Q, K[perm][:c], K[perm][c:])
        np.testing.assert_allclose(s_perm, s[perm], rtol=1e-11)
        # duplicating every query row doubles every score
        np.testing.assert_allclose(O.key_scores(np.concatenate([Q, Q]), Kc, Kk), 2 * s, rtol=1e-12)
        # a per-row constant shift of the logits changes nothing: extra channel that is
        # 1 in every key and arbitrary in each query
        extra = rng.standard_normal((R, 1)).astype(np.float32) * 4
        Q2 = np.concatenate([Q * math.sqrt((d + 1) / d), extra], axis=1)
        K2 = np.concatenate([K, np.ones((N, 1), np.float32)], axis=1)
        np.testing.assert_allclose(O.key_scores(Q2.astype(np.float64), K2[:c], K2[c:]), s, rtol=1e-6)


def pin_identity_when_budget_covers(O):
    rng = np.random.default_rng(12)
    Q = rng.standard_normal((4, 8)).astype(np.float32)
    Kc, Kk = rng.standard_normal((5, 8)).astype(np.float32), rng.standard_normal((6, 8)).astype(np.float32)
    Vc, Vk = rng.standard_normal((5, 8)).astype(np.float32), rng.standard_normal((6, 8)).astype(np.float32)
    for r in (11, 12, 1000):
        _, idx, Kn, Vn = O.step(Q, Kc, Vc, Kk, Vk, r)
        assert list(idx) == list(range(11))
        assert Kn.tobytes() == np.concatenate([Kc, Kk]).tobytes()
        assert Vn.tobytes() == np.concatenate([Vc, Vk]).tobytes()


def pin_tie_rule(O):
    s = np.array([0.5, 0.9, 0.5, 0.9, 0.5, 0.1], dtype=np.float32)
    assert list(O.top_r(s, 1)) == [1]
    assert list(O.top_r(s, 2)) == [1, 3]
    assert list(O.top_r(s, 3)) == [0, 1, 3]
    assert list(O.top_r(s, 4)) == [0, 1, 2, 3]
    assert list(O.top_r(s, 5)) == [0, 1, 2, 3, 4]
    assert O.top_r(s, 0).shape == (0,)
    # float32 input is ranked as float32 (no hidden rounding or widening effects)
    t = np.array([1.0, 1.0 + 2 ** -23, 1.0], dtype=np.float32)
    assert list(O.top_r(t, 2)) == [0, 1]


# --------------------------------------------------------------------- schedule

def pin_schedule_golden(O):
    with open(os.path.join(GOLDEN, "schedule_examples.txt")) as f:
        rows = [list(map(int, ln.split())) for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 4
    for n_cont, m, k, first, second, last, count in rows:
        rs = O.schedule(n_cont, m, k)
        assert len(rs) == count and rs[0] == first and rs[1] == second and rs[-1] == last
        sigma = n_cont / k
        c = 0
        for r in rs:                      # the paper's rule, increments m/sigma
            assert r == c + round(m / sigma)
            c = r


def pin_schedule_properties(O):
    for n_cont, m, k in [(1000, 256, 100), (2049, 2048, 64), (5, 8, 2), (4096, 512, 5000),
                         (777, 100, 777), (65536, 2048, 2048), (2048, 2048, 64), (3000, 7, 1)]:
        rs = O.schedule(n_cont, m, k)
        assert len(rs) == -(-n_cont // m)
        c = seen = 0
        for i, r in enumerate(rs):
            mi = min(m, n_cont - seen)
            seen += mi
            assert 0 <= r <= c + mi               # never more than the candidates
            assert r == min(c + mi, (min(k, n_cont) * seen) // n_cont)
            c = r
        assert rs[-1] == min(k, n_cont)
        assert all(b >= a for a, b in zip(rs, rs[1:]))    # monotone
        if k >= n_cont:                                   # no compression: keep everything seen
            assert rs == [min((i + 1) * m, n_cont) for i in range(len(rs))]
    assert O.schedule(0, 16, 4) == []


# --------------------------------------------------------------- chunk recurrence

def pin_single_chunk_is_one_shot(O):
    rng = np.random.default_rng(13)
    Q = rng.standard_normal((5, 8)).astype(np.float32)
    K = rng.standard_normal((40, 8)).astype(np.float32)
    V = rng.standard_normal((40, 8)).astype(np.float32)
    Kt, Vt, pos, hist = O.compress(Q, K, V, m=40, k=9)
    want = brute_top(brute_scores(Q, K[:0], K), 9)
    assert list(pos) == want and len(hist) == 1
    assert Kt.tobytes() == K[want].tobytes() and Vt.tobytes() == V[want].tobytes()


def pin_sigma_one_is_identity(O):
    rng = np.random.default_rng(14)
    Q = rng.standard_normal((3, 4)).astype(np.float32)
    K = rng.standard_normal((23, 4)).astype(np.float32)
    V = rng.standard_normal((23, 4)).astype(np.float32)
    for k in (23, 50):
        Kt, Vt, pos, _ = O.compress(Q, K, V, m=5, k=k)
        assert list(pos) == list(range(23))
        assert Kt.tobytes() == K.tobytes() and Vt.tobytes() == V.tobytes()


def pin_recurrence_brute_force(O):
    """Whole chunk loop against a pure-Python re-statement: at each step the
    candidates are the rows kept so far plus the new chunk, all re-scored."""
    rng = np.random.default_rng(15)
    Q = rng.standard_normal((4, 8)).astype(np.float32)
    K = rng.standard_normal((50, 8)).astype(np.float32)
    V = rng.standard_normal((50, 8)).astype(np.float32)
    m, k = 12, 10
    rs = [2, 4, 7, 9, 10]                 # floor(10 * seen / 50), seen = 12,24,36,48,50
    assert O.schedule(50, m, k) == rs
    kept = []
    for i, r in enumerate(rs):
        cand = kept + list(range(i * m, min((i + 1) * m, 50)))
        sc = brute_scores(Q, K[:0], K[cand])
        kept = [cand[j] for j in brute_top(sc, r)]
    Kt, Vt, pos, hist = O.compress(Q, K, V, m, k)
    assert list(pos) == kept and len(hist) == 5
    assert Kt.tobytes() == K[kept].tobytes() and Vt.tobytes() == V[kept].tobytes()


def pin_cached_row_can_be_evicted(O):
    # step 1 keeps row 0 (the only strong key of chunk 1); chunk 2 holds two stronger
    # keys, and with r = 2 the previously cached row must go.
    d = 4
    Q = np.array([[4.0, 0, 0, 0]])
    K = np.zeros((6, d))
    K[0, 0] = 1.0
    K[3, 0] = 3.0
    K[5, 0] = 2.0
    V = np.arange(24, dtype=np.float64).reshape(6, d)
    Kt, Vt, pos, hist = O.compress(Q, K, V, m=3, k=2, rs=[1, 2])
    assert list(hist[0][1]) == [0]
    assert list(pos) == [3, 5]
    assert Vt.tobytes() == V[[3, 5]].tobytes()


def pin_per_step_queries(O):
    # a different Q per step: step 2 ranks by its own Q, not by step 1's
    d = 2
    K = np.array([[2.0, 0], [0, 2.0], [2.0, 0], [0, 2.0]])
    V = K.copy()
    Qa, Qb = np.array([[5.0, 0]]), np.array([[0, 5.0]])
    _, _, pos, _ = O.compress([Qa, Qb], K, V, m=2, k=1, rs=[1, 1])
    assert list(pos) == [3]
    _, _, pos, _ = O.compress([Qa, Qa], K, V, m=2, k=1, rs=[1, 1])
    assert list(pos) == [0]


def pin_split_and_resume(O):
    rng = np.random.default_rng(16)
    Q = rng.standard_normal((3, 8)).astype(np.float32)
    K = rng.standard_normal((64, 8)).astype(np.float32)
    V = rng.standard_normal((64, 8)).astype(np.float32)
    rs = O.schedule(64, 16, 8)
    Kt, Vt, pos, _ = O.compress(Q, K, V, 16, 8)
    # run two steps, "save" the cache, continue with explicit step calls
    Kc, Vc, p2, _ = O.compress(Q, K[:32], V[:32], 16, 8, rs=rs[:2])
    for i in (2, 3):
        _, idx, Kc, Vc = O.step(Q, Kc, Vc, K[16 * i:16 * i + 16], V[16 * i:16 * i + 16], rs[i])
        p2 = np.concatenate([p2, np.arange(16 * i, 16 * i + 16)])[idx]
    assert list(p2) == list(pos) and Kc.tobytes() == Kt.tobytes() and Vc.tobytes() == Vt.tobytes()


# ------------------------------------------------------------ paper's worked example

def pin_reposition_example(O):
    with open(os.path.join(GOLDEN, "reposition_example.txt")) as f:
        rows = [list(map(int, ln.split())) for ln in f if ln.strip() and not ln.startswith("#")]
    ranking = [r[0] for r in rows]
    assert ranking == [3, 5, 0]
    assert O.reposition(ranking) == [r[1] for r in rows]


def golden_lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def pin_rope_zero_shift_is_identity(O):
    rng = np.random.default_rng(31)
    K = rng.standard_normal((5, 16)).astype(np.float32)
    for pairing in ("half", "interleaved"):
        out = O.rope_rotate(K, np.zeros(5), 10000.0, pairing)
        assert out.tobytes() == K.astype(np.float64).tobytes()


def pin_rope_closed_form(O):
    # d = 2: one pair, theta_0 = 1, so a shift by a turns (1, 0) into (cos a, sin a)
    # and (0, 1) into (-sin a, cos a), for any base and either pairing
    for pairing in ("half", "interleaved"):
        for a in (1.0, -2.5, 7.0):
            out = O.rope_rotate(np.array([[1.0, 0.0], [0.0, 1.0]], dtype=np.float32), [a, a], 123.0, pairing)
            want = np.array([[math.cos(a), math.sin(a)], [-math.sin(a), math.cos(a)]])
            assert np.abs(out - want).max() < 1e-15
    # theta_u = base^(-2u/d): with d = 4 and base 100 the second pair turns 10 times slower
    f = O.rope_frequencies(4, 100.0)
    assert abs(f[0] - 1.0) < 1e-15 and abs(f[1] - 0.1) < 1e-15
    out = O.rope_rotate(np.array([[0.0, 1.0, 0.0, 0.0]], dtype=np.float32), [5.0], 100.0, "half")
    # half pairing: channel 1 pairs with channel 3 and is pair u = 1
    assert np.abs(out - np.array([[0.0, math.cos(0.5), 0.0, math.sin(0.5)]])).max() < 1e-15
    out = O.rope_rotate(np.array([[0.0, 0.0, 1.0, 0.0]], dtype=np.float32), [5.0], 100.0, "interleaved")
    # interleaved pairing: channel 2 pairs with channel 3 and is pair u = 1
    assert np.abs(out - np.array([[0.0, 0.0, math.cos(0.5), math.sin(0.5)]])).max() < 1e-15


def pin_rope_against_complex_multiplication(O):
    rng = np.random.default_rng(32)
    d, n, base = 32, 7, 500000.0
    K = rng.standard_normal((n, d)).astype(np.float32)
    delta = rng.integers(-3000, 3000, n)
    theta = np.array([base ** (-2.0 * u / d) for u in range(d // 2)])
    for pairing in ("half", "interleaved"):
        out = O.rope_rotate(K, delta, base, pairing)
        K64 = K.astype(np.float64)
        a, b = (K64[:, :d // 2], K64[:, d // 2:]) if pairing == "half" else (K64[:, 0::2], K64[:, 1::2])
        z = (a + 1j * b) * np.exp(1j * delta[:, None] * theta[None, :])
        got = (out[:, :d // 2] + 1j * out[:, d // 2:]) if pairing == "half" else (out[:, 0::2] + 1j * out[:, 1::2])
        assert np.abs(got - z).max() < 1e-12


def pin_rope_shifts_add_and_keep_relative_positions(O):
    rng = np.random.default_rng(33)
    d, base = 64, 10000.0
    q = rng.standard_normal((1, d)).astype(np.float32)
    k = rng.standard_normal((1, d)).astype(np.float32)
    for pairing in ("half", "interleaved"):
        once = O.rope_rotate(k, [17 - 40], base, pairing)
        twice = O.rope_rotate(O.rope_rotate(k, [-30], base, pairing), [7], base, pairing)
        assert np.abs(once - twice).max() < 1e-12
        # pair norms do not change
        n0 = (k.astype(np.float64) ** 2).sum()
        assert abs((once ** 2).sum() - n0) < 1e-10
        # a key encoded at position 40 and moved to 17 meets a query at position 20 exactly
        # as a key that was encoded at 17 in the first place: only differences count
        k40 = O.rope_rotate(k, [40], base, pairing)
        k17 = O.rope_rotate(k, [17], base, pairing)
        q20 = O.rope_rotate(q, [20], base, pairing)
        moved = O.rope_rotate(k40, [17 - 40], base, pairing)
        assert np.abs(moved - k17).max() < 1e-12
        assert abs((q20 * moved).sum() - (O.rope_rotate(q, [3], base, pairing) * k.astype(np.float64)).sum()) < 1e-10


def pin_kept_slots_worked_example(O):
    # Managing the Cache: cache [0..5], relevance ranking [3, 5, 0]
    moves = {}
    for line in golden_lines("reposition_example.txt"):
        e, mv = line.split()
        moves[int(e)] = int(mv)
    scores = np.array([0.3, 0.0, 0.01, 0.9, 0.02, 0.5])
    idx = O.top_r(scores, 3)
    assert idx.tolist() == [0, 3, 5]
    slots = O.kept_slots(idx, scores, "rank")
    assert slots.tolist() == [2, 0, 1]
    assert {int(i): int(s - i) for i, s in zip(idx, slots)} == moves
    assert O.kept_slots(idx, scores, "ascending").tolist() == [0, 1, 2]
    # equal scores keep their index order
    assert O.kept_slots(np.array([1, 2, 4]), np.array([0, .5, .5, 0, .5]), "rank").tolist() == [0, 1, 2]


def pin_compact_repositioned(O):
    rng = np.random.default_rng(34)
    d, c, m = 8, 4, 5
    Kc, Kk = rng.standard_normal((c, d)).astype(np.float32), rng.standard_normal((m, d)).astype(np.float32)
    Vc, Vk = rng.standard_normal((c, d)).astype(np.float32), rng.standard_normal((m, d)).astype(np.float32)
    scores = rng.random(c + m)
    idx = O.top_r(scores, 4)
    allK, allV = np.concatenate([Kc, Kk]), np.concatenate([Vc, Vk])
    # no rotation, ascending: the plain compaction
    K0, V0, s0 = O.compact_repositioned(idx, scores, Kc, Kk, Vc, Vk, 1e4, None, "ascending")
    assert K0.tobytes() == allK[idx].astype(np.float64).tobytes() and V0.tobytes() == allV[idx].tobytes()
    # rank order: slot 0 holds the best candidate, values travel with their keys, and
    # each key is turned by (slot - old index) positions, checked row by row
    K1, V1, s1 = O.compact_repositioned(idx, scores, Kc, Kk, Vc, Vk, 1e4, "half", "rank")
    best = int(idx[np.argmax(scores[idx])])
    assert V1[0].tobytes() == allV[best].tobytes()
    assert sorted(s1.tolist()) == list(range(4))
    for t, j in enumerate(idx):
        want = O.rope_rotate(allK[j:j + 1], [int(s1[t]) - int(j)], 1e4, "half")[0]
        assert np.abs(K1[s1[t]] - want).max() < 1e-15
        assert V1[s1[t]].tobytes() == allV[j].tobytes()
    # ascending order never moves a key to a later position
    K2, V2, s2 = O.compact_repositioned(idx, scores, Kc, Kk, Vc, Vk, 1e4, "interleaved", "ascending")
    assert ((s2 - idx) <= 0).all()


def pin_paper_exact_denominator(O):
    """The prompt-guided sub-matrix as the model forms it: softmax over context AND
    (causally) prompt keys, then the context columns.  Built here with an explicit
    mask and scipy's softmax."""
    from scipy.special import softmax
    rng = np.random.default_rng(41)
    d, G, nq, c, m = 16, 3, 5, 4, 7
    Q = rng.standard_normal((G * nq, d)).astype(np.float32)
    Kq = rng.standard_normal((nq, d)).astype(np.float32)
    Kc = rng.standard_normal((c, d)).astype(np.float32)
    Kk = rng.standard_normal((m, d)).astype(np.float32)
    allk = np.concatenate([Kc, Kk, Kq]).astype(np.float64)
    S = Q.astype(np.float64) @ allk.T / math.sqrt(d)
    for row in range(G * nq):
        t = row % nq
        S[row, c + m + t + 1:] = -np.inf          # prompt keys after the token itself
    A = softmax(S, axis=1)
    want = A[:, :c + m].sum(axis=0)
    extra = O.prompt_lse(Q, Kq, G)
    got = O.key_scores(Q, Kc, Kk, lse_extra=extra)
    assert np.abs(got - want).max() < 1e-13
    # the prompt's share is gone from the total: sum < R, and by exactly that share
    assert abs(got.sum() - (G * nq - A[:, c + m:].sum())) < 1e-12
    # first token of every head sees only its own key among the prompt keys
    for g in range(G):
        q0 = Q[g * nq].astype(np.float64)
        assert abs(extra[g * nq] - q0 @ Kq[0].astype(np.float64) / math.sqrt(d)) < 1e-13
    # no extra keys (lse_extra = -inf) is the default reading
    base = O.key_scores(Q, Kc, Kk)
    same = O.key_scores(Q, Kc, Kk, lse_extra=np.full(G * nq, -np.inf))
    assert np.abs(base - same).max() < 1e-15
    # one prompt row: the extra keys scale every score by one factor, ranking unchanged
    one = O.key_scores(Q[:1], Kc, Kk, lse_extra=extra[:1])
    ref = O.key_scores(Q[:1], Kc, Kk)
    assert np.abs(one / ref - (one / ref)[0]).max() < 1e-13 and (one < ref).all()


def pin_layer_wise_selection(O):
    rng = np.random.default_rng(51)
    d, H, nq, c, m, r = 8, 3, 2, 3, 5, 4
    Qs = [rng.standard_normal((nq, d)).astype(np.float32) for _ in range(H)]
    Kc = [rng.standard_normal((c, d)).astype(np.float32) for _ in range(H)]
    Kk = [rng.standard_normal((m, d)).astype(np.float32) for _ in range(H)]
    Vc = [rng.standard_normal((c, d)).astype(np.float32) for _ in range(H)]
    Vk = [rng.standard_normal((m, d)).astype(np.float32) for _ in range(H)]
    per_head, total, idx, Ks, Vs = O.step_layer(Qs, Kc, Vc, Kk, Vk, r)
    # brute force: plain loops over heads, prompt rows and keys
    want = [0.0] * (c + m)
    for h in range(H):
        keys = [list(map(float, row)) for row in np.concatenate([Kc[h], Kk[h]])]
        for i in range(nq):
            q = list(map(float, Qs[h][i]))
            logits = [sum(a * b for a, b in zip(q, k)) / math.sqrt(d) for k in keys]
            mx = max(logits)
            e = [math.exp(x - mx) for x in logits]
            z = sum(e)
            for j in range(c + m):
                want[j] += e[j] / z
    assert max(abs(a - b) for a, b in zip(total, want)) < 1e-12
    assert abs(total.sum() - H * nq) < 1e-12
    order = sorted(range(c + m), key=lambda j: (-want[j], j))[:r]
    assert idx.tolist() == sorted(order)
    for h in range(H):      # every head keeps the SAME positions of its own rows
        allk, allv = np.concatenate([Kc[h], Kk[h]]), np.concatenate([Vc[h], Vk[h]])
        assert Ks[h].tobytes() == allk[idx].tobytes() and Vs[h].tobytes() == allv[idx].tobytes()
    # heads that disagree: head 0 puts all its weight on key 0, heads 1 and 2 put 0.6 of
    # theirs on key 1 and the rest on key 2; the layer keeps key 1 (1.2) over key 0 (1.0),
    # although head 0 alone would keep key 0
    big = 60.0
    K = np.eye(3, 4, dtype=np.float32) * big
    q0 = np.array([[1, 0, 0, 0]], dtype=np.float32) * big
    a = math.log(0.6 / 0.4) * 2.0 / big ** 2  # logits of keys 1, 2 differ by ln(0.6/0.4): sqrt(d) = 2
    q1 = np.array([[0, 1.0 + a / 2, 1.0 - a / 2, 0]], dtype=np.float32) * big
    ph, tot, idx1, _, _ = O.step_layer([q0, q1, q1], [K[:0]] * 3, [K[:0]] * 3, [K] * 3, [K] * 3, 1)
    assert abs(tot[0] - 1.0) < 1e-6 and abs(tot[1] - 1.2) < 1e-3 and abs(tot[2] - 0.8) < 1e-3
    assert idx1.tolist() == [1] and O.top_r(ph[0], 1).tolist() == [0]
    # identical heads: the layer's choice is each head's choice
    phs, tots, idxs, _, _ = O.step_layer([Qs[0]] * 4, [Kc[0]] * 4, [Vc[0]] * 4, [Kk[0]] * 4, [Vk[0]] * 4, r)
    assert idxs.tolist() == O.top_r(phs[0], r).tolist()
    assert np.abs(tots - 4 * phs[0]).max() < 1e-13


def pin_constant_budget_schedule(O):
    # every step keeps min(k, candidates): C4's shape (131072 tokens, chunks of 4096, k = 1408)
    rs = O.schedule(131072, 4096, 1408, constant_budget=True)
    assert rs == [1408] * 32
    keys = sum((rs[i - 1] if i else 0) + 4096 for i in range(32))
    assert keys == 32 * 4096 + 31 * 1408          # = 174 720 keys scored per problem
    assert O.schedule(1000, 300, 500, constant_budget=True) == [300, 500, 500, 500]
    assert O.schedule(1000, 300, 5000, constant_budget=True) == [300, 600, 900, 1000]
    assert O.schedule(131072, 4096, 1408)[-1] == 1408 and O.schedule(131072, 4096, 1408)[0] == 44


def pin_conditioned_on_document_rows(O):
    from scipy.special import softmax
    rng = np.random.default_rng(61)
    d, G, nq, c, m = 8, 2, 3, 4, 6
    N = c + m
    Qp = rng.standard_normal((G * nq, d)).astype(np.float32)
    Qd = rng.standard_normal((G * m, d)).astype(np.float32)
    Kc = rng.standard_normal((c, d)).astype(np.float32)
    Kk = rng.standard_normal((m, d)).astype(np.float32)
    K = np.concatenate([Kc, Kk]).astype(np.float64)
    # scipy on the explicitly masked matrix, rows weighted by (visible keys) / N
    S = Qd.astype(np.float64) @ K.T / math.sqrt(d)
    vis = np.array([c + (row % m) + 1 for row in range(G * m)])
    for row in range(G * m):
        S[row, vis[row]:] = -np.inf
    A = softmax(S, axis=1) * (vis / N)[:, None]
    want_doc = A.sum(axis=0)
    got_doc = O.key_scores_conditioned(None, Qd, Kc, Kk, G)
    assert np.abs(got_doc - want_doc).max() < 1e-13
    # pure-Python loops
    brute = [0.0] * N
    for row in range(G * m):
        i = row % m
        q = list(map(float, Qd[row]))
        logits = [sum(a * b for a, b in zip(q, map(float, K[j]))) / math.sqrt(d) for j in range(c + i + 1)]
        mx = max(logits)
        e = [math.exp(x - mx) for x in logits]
        z = sum(e)
        for j in range(c + i + 1):
            brute[j] += e[j] / z * (c + i + 1) / N
    assert max(abs(a - b) for a, b in zip(got_doc, brute)) < 1e-12
    # both row sets: the sum of the two; prompt rows carry weight 1
    both = O.key_scores_conditioned(Qp, Qd, Kc, Kk, G)
    assert np.abs(both - (want_doc + O.key_scores(Qp, Kc, Kk))).max() < 1e-13
    assert np.abs(O.key_scores_conditioned(Qp, None, Kc, Kk, G) - O.key_scores(Qp, Kc, Kk)).max() < 1e-15
    # all scores add up to the sum of the row weights
    assert abs(got_doc.sum() - (vis / N).sum()) < 1e-12
    # no cache: the same by hand over the chunk alone
    first = O.key_scores_conditioned(None, Qd, Kc[:0], Kk, G)
    only_first_rows = np.zeros(m)
    S0 = Qd.astype(np.float64) @ Kk.astype(np.float64).T / math.sqrt(d)
    for row in range(G * m):
        i = row % m
        s = S0[row, :i + 1]
        e = np.exp(s - s.max())
        only_first_rows[:i + 1] += e / e.sum() * (i + 1) / m
    assert np.abs(first - only_first_rows).max() < 1e-13
    # closed form: a chunk of one token sees only itself and gives its key weight 1
    one = O.key_scores_conditioned(None, Qd[:1], Kc[:0], Kk[:1], 1)
    assert abs(one[0] - 1.0) < 1e-15
    # causality: changing the LAST chunk key changes nothing that earlier chunk rows give:
    # with only the first m-1 tokens' rows, the result is the same for either last key
    Kk2 = Kk.copy()
    Kk2[-1] += 3.0
    rows_but_last = np.array([r for r in range(G * m) if r % m != m - 1])
    def partial(Kx):
        Kall = np.concatenate([Kc, Kx]).astype(np.float64)
        out = np.zeros(N)
        Sx = Qd.astype(np.float64) @ Kall.T / math.sqrt(d)
        for row in rows_but_last:
            v = c + (row % m) + 1
            e = np.exp(Sx[row, :v] - Sx[row, :v].max())
            out[:v] += e / e.sum() * v / N
        return out
    last_rows_a = O.key_scores_conditioned(None, Qd, Kc, Kk, G) - partial(Kk)
    assert np.abs(partial(Kk) - partial(Kk2)).max() < 1e-15
    assert np.abs(last_rows_a).max() > 1e-3 and (last_rows_a >= -1e-15).all()


ALL_PINS = [v for k, v in sorted(globals().items()) if k.startswith("pin_") and callable(v)]
