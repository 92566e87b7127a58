"""CPU oracle for Finch's prompt-guided top-r selection (arxiv 2408.00167).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition the HIP path is
checked against.  It is imported by tests/, by `__graft_entry__.smoke()` and by
the `cpu_baseline` leg of bench.py, and by nothing else; it shares no code with
the HIP library and imports nothing from it.

Everything is fp64 numpy.  Inputs are taken exactly as stored: float32 arrays are
widened, bfloat16 arrays arrive as uint16 bit patterns and are widened exactly, so
products are exact and only summation order can differ from other
implementations.  One *problem* is one (request, layer, KV head): Q holds the
R = G * n_que prompt rows of the G query heads sharing that KV head, stacked.

Steps follow the paper's Method section, "Prompt-Guided Layer-wise top r position
selection" and "Managing the Cache", with these readings where the text leaves a
choice (each is listed in the design notes of the repository):
  * softmax denominator: over the c + m context keys (cache then chunk) only;
  * head sum: over the G query heads of one KV group (the rows stacked in Q);
  * the normalisation factor count(A != 0)/(m + c) is one positive constant for
    all keys of a step (every prompt row sees every context key), so it is
    dropped: sum_j score_j == R;
  * d_k in the scale is the head dimension;
  * top-r ties go to the lowest index, kept rows stay in ascending index order;
  * r schedule: r_i = min(c_{i-1} + m_i, floor(k * seen_i / n_cont)), which equals
    the paper's r_{it+1} = m_{it+1}/sigma + c_it whenever m/sigma is an integer
    and ends at r = k.

Pins (tests/test_oracle_*.py, all `-m "not gpu"`): closed-form softmax values on
one-hot constructions, uniform scores for identical keys, R = 1 reducing to an
argsort of raw dot products, scipy's softmax/logsumexp on random inputs,
pure-Python brute force (explicit full matrix + full sort) on tiny inputs, the
invariants (rows sum to 1, sum of scores = R, exactly min(r, N) kept, ascending,
r >= N is the identity), the schedule's closed forms, single-chunk == one-shot,
sigma = 1 == identity, and planted-mistake tests showing that a dropped scale, a
transposed operand, a wrong axis, a wrong tie rule or a wrong concatenation order
each break at least one pin.  `reposition` is pinned by the paper's worked example.

Re-positioning of the kept keys (Managing the Cache: the positional embedding of a
kept pair is adjusted to the slot it moves to; for rotary embeddings that is a
rotation by the slot difference): `rope_rotate`, `kept_slots`,
`compact_repositioned`.  Readings: a candidate's current position is its index in
[cache ; chunk]; its new position is its slot in the new cache - slot t for the
t-th kept index in ascending order, or, as in the paper's worked example, the
rank of its score among the kept ones (highest first, ties to the lower index);
the rotary pairing is either (u, u + d/2) ("half", the Llama layout the paper
names) or (2u, 2u+1) ("interleaved", RoFormer's own); theta_u = base^(-2u/d).
The paper-exact denominator (`prompt_lse`, `key_scores(..., lse_extra=...)`): in
the model the prompt rows' softmax also runs over the prompt's own keys, causally;
the default reading leaves them out.  Pinned by the explicit attention matrix over
[context ; prompt] columns with the causal mask written out, softmaxed by scipy,
from which the context columns are cut.

Layer-wise selection as the paper words it (`layer_scores`, `step_layer`: the
scores of all heads of a layer are summed and one index set serves every head) and
the constant-budget schedule (`schedule(..., constant_budget=True)`).  Pinned by a
pure-Python triple loop over heads, rows and keys, by a construction in which the
heads disagree and the layer's choice is known in closed form, by H identical heads
reproducing the single-head choice, and by closed forms of the schedule.

Conditioning on the chunk's own rows (`key_scores_conditioned`: the paper's
ablation, rows = chunk tokens with the causal mask, alone or together with the
prompt rows, and the Method's normalisation read per row).  Pinned by a pure-Python
loop with the mask written out, by scipy's softmax on the -inf-masked matrix, by
closed forms (first chunk token, sum of all scores = sum of the row weights), by
causality (a later key cannot change what earlier rows give) and by the reduction to
`key_scores` when there are no chunk rows.

Pins: a rotation by zero is the identity bit for bit, rotations add up, pair norms
are kept, dot products of two rotated vectors depend only on the difference of
their positions, the closed form (1, 0) -> (cos a, sin a), numpy's complex
multiplication as an independent statement of the same rotation, and the worked
example's moves (-3, -4, +2) for the slots.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

__all__ = ["widen", "attention_weights", "key_scores", "top_r", "gather_rows",
           "step", "schedule", "compress", "reposition", "rope_frequencies", "rope_rotate",
           "kept_slots", "compact_repositioned", "prompt_lse", "layer_scores", "step_layer", "key_scores_conditioned"]


def widen(x: np.ndarray) -> np.ndarray:
    """Stored values -> float64, exactly.  uint16 is read as bfloat16 bits."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported storage dtype {x.dtype}")


def attention_weights(Q: np.ndarray, K: np.ndarray) -> np.ndarray:
    """softmax(Q K^T / sqrt(d_k)) row by row (Background, attention equation).

    Q is [R][d], K is [N][d]; returns the R x N matrix of weights, each row a
    distribution over the N keys.
    """
    Q = widen(Q)
    K = widen(K)
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(float(d))
    if S.shape[1] == 0:
        return S
    mx = S.max(axis=1, keepdims=True)
    E = np.exp(S - mx)
    Z = E.sum(axis=1, keepdims=True)
    return E / Z


def key_scores(Q: np.ndarray, K_cache: np.ndarray, K_chunk: np.ndarray,
               lse_extra: Optional[np.ndarray] = None) -> np.ndarray:
    """One relevance score per context key (Method: sum over heads, prompt-guided
    sub-matrix, aggregation over prompt rows).

    Keys are ordered cache rows first, then chunk rows.  Because Q already stacks
    the prompt rows of every head of the group, the head sum and the sum over
    prompt tokens are one column sum of the weight matrix.

    lse_extra (one value per row of Q, natural log) widens every row's softmax by
    keys that are not candidates: the row's weights over the context keys become
    exp(s_ij) / (sum_j exp(s_ij) + exp(lse_extra_i)).  With `prompt_lse` this gives
    the prompt-guided sub-matrix exactly as the model computes it, where a prompt
    token also attends, causally, to the prompt itself.
    """
    K = np.concatenate([np.asarray(K_cache), np.asarray(K_chunk)], axis=0)
    P = attention_weights(Q, K)
    if lse_extra is not None and P.shape[1] > 0:
        Qw, Kw = widen(Q), widen(K)
        S = (Qw @ Kw.T) / math.sqrt(float(Qw.shape[1]))
        mx = S.max(axis=1)
        lse_ctx = mx + np.log(np.exp(S - mx[:, None]).sum(axis=1))
        share = 1.0 / (1.0 + np.exp(np.asarray(lse_extra, dtype=np.float64) - lse_ctx))
        P = P * share[:, None]
    return P.sum(axis=0)


def prompt_lse(Q: np.ndarray, K_que: np.ndarray, group: int) -> np.ndarray:
    """log sum exp of each prompt row's logits over the prompt's own keys under the
    causal mask (Method: the prompt follows the context in the model's input, so a
    prompt token sees the context and the prompt tokens up to itself).  Q stacks
    the `group` heads, n_que rows each; row g*n_que + t is token t and sees prompt
    keys 0..t of K_que [n_que][d].  Natural log, float64.
    """
    Qw, Kw = widen(Q), widen(K_que)
    n_que = Kw.shape[0]
    assert Qw.shape[0] == group * n_que
    S = (Qw @ Kw.T) / math.sqrt(float(Qw.shape[1]))
    out = np.empty(Qw.shape[0], dtype=np.float64)
    for row in range(Qw.shape[0]):
        t = row % n_que
        s = S[row, :t + 1]
        out[row] = s.max() + math.log(np.exp(s - s.max()).sum())
    return out


def top_r(scores: np.ndarray, r: int) -> np.ndarray:
    """Indices of the r highest scores, ties to the lowest index, returned in
    ascending index order (Method: t = top-r(A_agg, r)).  r is clamped to
    [0, N].  Works on whatever precision `scores` has, without converting it.
    """
    scores = np.asarray(scores)
    n = scores.shape[0]
    r = max(0, min(int(r), n))
    order = np.argsort(-scores, kind="stable")     # descending, equal scores by index
    return np.sort(order[:r]).astype(np.int32)


def gather_rows(idx: np.ndarray, cache: np.ndarray, chunk: np.ndarray) -> np.ndarray:
    """Rows idx of [cache ; chunk], copied bit for bit (Managing the Cache)."""
    both = np.concatenate([np.asarray(cache), np.asarray(chunk)], axis=0)
    return both[np.asarray(idx, dtype=np.int64)].copy()


def step(Q, K_cache, V_cache, K_chunk, V_chunk, r: int):
    """One prefill step for one problem: score, select, compact.

    Returns (scores fp64 [c+m], idx int32 [min(r, c+m)] ascending, K', V').
    """
    scores = key_scores(Q, K_cache, K_chunk)
    idx = top_r(scores, r)
    return scores, idx, gather_rows(idx, K_cache, K_chunk), gather_rows(idx, V_cache, V_chunk)


def schedule(n_cont: int, m: int, k: int, constant_budget: bool = False) -> List[int]:
    """Rows kept after each chunk step (Method: the r update rule; the last value
    is the target size k, or n_cont if the budget is not smaller).  With
    `constant_budget` every step keeps the full budget k as soon as that many
    candidates exist ("top-k under the budget" read literally) instead of growing
    r in proportion to the tokens seen."""
    if n_cont <= 0:
        return []
    out: List[int] = []
    c = 0
    seen = 0
    k = min(int(k), int(n_cont))
    while seen < n_cont:
        mi = min(m, n_cont - seen)
        seen += mi
        r = min(c + mi, k if constant_budget else (k * seen) // n_cont)
        out.append(r)
        c = r
    return out


def compress(Q, K_doc: np.ndarray, V_doc: np.ndarray, m: int, k: int,
             rs: Optional[Sequence[int]] = None):
    """The chunk loop for one problem (Method: Document Segmentation + Compression
    Output).  Q is either one [R][d] block used at every step or a sequence with
    one block per step.

    Returns (K~, V~, positions, history) where positions[t] is the document index
    of kept row t and history is the per-step list of (scores, idx).
    """
    K_doc = np.asarray(K_doc)
    V_doc = np.asarray(V_doc)
    n_cont = K_doc.shape[0]
    rs = list(schedule(n_cont, m, k) if rs is None else rs)
    Kc, Vc = K_doc[:0].copy(), V_doc[:0].copy()
    pos = np.zeros(0, dtype=np.int64)
    history: List[Tuple[np.ndarray, np.ndarray]] = []
    for i, r in enumerate(rs):
        lo, hi = i * m, min((i + 1) * m, n_cont)
        q = Q[i] if isinstance(Q, (list, tuple)) else Q
        scores, idx, Kn, Vn = step(q, Kc, Vc, K_doc[lo:hi], V_doc[lo:hi], r)
        pos = np.concatenate([pos, np.arange(lo, hi, dtype=np.int64)])[idx]
        Kc, Vc = Kn, Vn
        history.append((scores, idx))
    return Kc, Vc, pos, history


def reposition(ranking: Sequence[int]) -> List[int]:
    """Signed slot moves of the kept cache entries when they are re-packed in
    relevance-rank order (Managing the Cache, worked example): entry at old slot
    ranking[t] goes to new slot t; negative = towards the start.
    """
    return [t - int(old) for t, old in enumerate(ranking)]


def rope_frequencies(d: int, base: float) -> np.ndarray:
    """theta_u = base^(-2u/d), u = 0 .. d/2 - 1: the rotary embedding's angle per
    position step of channel pair u (RoFormer, as used by Llama 2, which the
    paper's Managing the Cache names)."""
    u = np.arange(d // 2, dtype=np.float64)
    return np.power(float(base), -2.0 * u / float(d))


def rope_rotate(K: np.ndarray, delta: np.ndarray, base: float, pairing: str) -> np.ndarray:
    """Rows of K moved by delta[t] positions (Managing the Cache: the cosine and
    sine needed for rotating to earlier or later positions): channel pair u of row
    t is turned by the angle delta[t] * theta_u.  Returns float64; rows with
    delta == 0 come back unchanged.
    """
    X = widen(K)
    n, d = X.shape
    ang = np.asarray(delta, dtype=np.float64)[:, None] * rope_frequencies(d, base)[None, :]
    cs, sn = np.cos(ang), np.sin(ang)
    if pairing == "half":
        a, b = X[:, :d // 2], X[:, d // 2:]
        out = np.concatenate([a * cs - b * sn, b * cs + a * sn], axis=1)
    elif pairing == "interleaved":
        a, b = X[:, 0::2], X[:, 1::2]
        out = np.empty_like(X)
        out[:, 0::2] = a * cs - b * sn
        out[:, 1::2] = b * cs + a * sn
    else:
        raise ValueError(pairing)
    return out


def kept_slots(idx: np.ndarray, scores: np.ndarray, order: str) -> np.ndarray:
    """New cache slot of each kept candidate idx[t] (idx ascending).  "ascending":
    slot t.  "rank": the kept ones packed by relevance, highest score first, equal
    scores by index (Managing the Cache, worked example)."""
    idx = np.asarray(idx, dtype=np.int64)
    if order == "ascending":
        return np.arange(idx.shape[0], dtype=np.int64)
    if order != "rank":
        raise ValueError(order)
    by_rank = np.argsort(-np.asarray(scores)[idx], kind="stable")   # kept entry at each slot
    slots = np.empty(idx.shape[0], dtype=np.int64)
    slots[by_rank] = np.arange(idx.shape[0], dtype=np.int64)
    return slots


def compact_repositioned(idx, scores, K_cache, K_chunk, V_cache, V_chunk, base: float,
                         pairing: Optional[str], order: str):
    """The new cache with re-positioned keys: candidate idx[t] goes to slot
    kept_slots(...)[t]; its key is rotated by (slot - idx[t]) positions (not at all
    if `pairing` is None), its value is copied.  Returns (K' float64, V' as
    stored, slots)."""
    idx = np.asarray(idx, dtype=np.int64)
    slots = kept_slots(idx, scores, order)
    Ksel = gather_rows(idx, K_cache, K_chunk)
    Vsel = gather_rows(idx, V_cache, V_chunk)
    Krot = widen(Ksel) if pairing is None else rope_rotate(Ksel, slots - idx, base, pairing)
    Kout = np.empty_like(Krot)
    Vout = np.empty_like(Vsel)
    Kout[slots] = Krot
    Vout[slots] = Vsel
    return Kout, Vout, slots


def layer_scores(per_head: Sequence[np.ndarray]) -> np.ndarray:
    """The paper's layer-wise aggregate (Method: "Sum over heads" - the attention
    of ALL heads of a layer is added up before one top-r per layer): the per-key
    scores of the layer's KV heads, each already summed over its own query heads
    and prompt rows, added up head by head."""
    total = np.zeros_like(np.asarray(per_head[0], dtype=np.float64))
    for s in per_head:
        total = total + np.asarray(s, dtype=np.float64)
    return total


def step_layer(Qs, K_caches, V_caches, K_chunks, V_chunks, r: int, lse_extras=None):
    """One prefill step of one layer with the paper's layer-wise selection: every KV
    head h (own Q block, own keys and values, the same c and m) is scored, the
    scores are summed over the heads, ONE index set is chosen and every head keeps
    those positions.  Returns (per-head scores, layer scores, idx, [K'_h], [V'_h])."""
    H = len(Qs)
    per_head = [key_scores(Qs[h], K_caches[h], K_chunks[h],
                           None if lse_extras is None else lse_extras[h]) for h in range(H)]
    total = layer_scores(per_head)
    idx = top_r(total, r)
    return (per_head, total, idx,
            [gather_rows(idx, K_caches[h], K_chunks[h]) for h in range(H)],
            [gather_rows(idx, V_caches[h], V_chunks[h]) for h in range(H)])


def key_scores_conditioned(Q_prompt, Q_doc, K_cache: np.ndarray, K_chunk: np.ndarray, group: int,
                           lse_extra: Optional[np.ndarray] = None) -> np.ndarray:
    """Scores when the rows of the attention matrix are not (only) the prompt's (the
    paper's ablation of the conditioning: self-attention of the document chunk, or
    of chunk and prompt together, instead of the prompt alone), with the Method's
    normalisation step.

    The model's input is [cache ; chunk ; prompt].  Q_doc [group * m][d] stacks, head
    by head, the queries of the m chunk tokens; chunk token i (position c + i) sees
    the cache and the chunk keys up to itself: c + i + 1 keys.  Q_prompt
    [group * n_que][d] as in `key_scores` sees all c + m context keys.  Either may be
    None.  Every row is a softmax over the keys it sees; the normalisation multiplies
    row i by (keys row i sees) / (m + c) - read per row: it is what offsets the
    thinner spread of rows that see more keys, and it is 1 for prompt rows - and
    the score of key j is the sum over the rows that see it.
    """
    K = widen(np.concatenate([np.asarray(K_cache), np.asarray(K_chunk)], axis=0))
    c, m = np.asarray(K_cache).shape[0], np.asarray(K_chunk).shape[0]
    N = c + m
    total = np.zeros(N, dtype=np.float64)
    if Q_prompt is not None:
        total += key_scores(Q_prompt, K_cache, K_chunk, lse_extra)
    if Q_doc is not None and m > 0:
        Qd = widen(Q_doc)
        assert Qd.shape[0] == group * m
        S = (Qd @ K.T) / math.sqrt(float(Qd.shape[1]))
        for row in range(group * m):
            i = row % m
            vis = c + i + 1
            s = S[row, :vis]
            e = np.exp(s - s.max())
            total[:vis] += (e / e.sum()) * (vis / float(N))
    return total
