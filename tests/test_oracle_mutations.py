"""Planted mistakes: each plausible slip in the oracle must break at least one pin.

The oracle's source text is edited on the CPU, loaded as a throw-away module, and
the full pin list is run against it.  Nothing here touches the GPU.
"""
import os
import types

import pytest

from tests import oracle_pins

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                   "oracle", "finch_oracle.py")

MUTATIONS = {
    "doc_rows_not_causal": ("            vis = c + i + 1\n", "            vis = N\n"),
    "doc_rows_exclude_self": ("            vis = c + i + 1\n", "            vis = c + i\n"),
    "doc_rows_token_major": ("            i = row % m\n            vis", "            i = row // group\n            vis"),
    "doc_rows_not_normalised": ("total[:vis] += (e / e.sum()) * (vis / float(N))", "total[:vis] += (e / e.sum())"),
    "doc_rows_normalised_inversely": ("total[:vis] += (e / e.sum()) * (vis / float(N))", "total[:vis] += (e / e.sum()) * (float(N) / vis)"),
    "layer_keeps_first_head_only": ("for s in per_head:\n        total = total + np.asarray(s, dtype=np.float64)",
                                    "for s in per_head[:1]:\n        total = total + np.asarray(s, dtype=np.float64)"),
    "layer_mean_of_maxima": ("    idx = top_r(total, r)\n    return (per_head", "    idx = top_r(per_head[0], r)\n    return (per_head"),
    "layer_values_from_one_head": ("[gather_rows(idx, V_caches[h], V_chunks[h]) for h in range(H)])",
                                   "[gather_rows(idx, V_caches[0], V_chunks[0]) for h in range(H)])"),
    "constant_budget_ignored": ("k if constant_budget else (k * seen) // n_cont", "(k * seen) // n_cont"),
    "extra_keys_not_causal": ("s = S[row, :t + 1]", "s = S[row, :]"),
    "extra_keys_exclude_self": ("s = S[row, :t + 1]", "s = S[row, :max(t, 1)]"),
    "extra_rows_token_major": ("t = row % n_que\n        s = S[row", "t = row // group\n        s = S[row"),
    "extra_share_inverted": ("share = 1.0 / (1.0 + np.exp(np.asarray(lse_extra, dtype=np.float64) - lse_ctx))",
                             "share = 1.0 / (1.0 + np.exp(lse_ctx - np.asarray(lse_extra, dtype=np.float64)))"),
    "extra_share_ignored": ("P = P * share[:, None]", "P = P"),
    "rope_sine_sign": ("out = np.concatenate([a * cs - b * sn, b * cs + a * sn], axis=1)",
                       "out = np.concatenate([a * cs + b * sn, b * cs - a * sn], axis=1)"),
    "rope_interleaved_sine_sign": ("out[:, 0::2] = a * cs - b * sn\n        out[:, 1::2] = b * cs + a * sn",
                                   "out[:, 0::2] = a * cs + b * sn\n        out[:, 1::2] = b * cs - a * sn"),
    "rope_pairings_swapped": ("if pairing == \"half\":\n        a, b = X[:, :d // 2], X[:, d // 2:]",
                              "if pairing == \"interleaved\":\n        a, b = X[:, :d // 2], X[:, d // 2:]"),
    "rope_frequency_exponent": ("return np.power(float(base), -2.0 * u / float(d))",
                                "return np.power(float(base), -1.0 * u / float(d))"),
    "rope_frequency_sign": ("return np.power(float(base), -2.0 * u / float(d))",
                            "return np.power(float(base), 2.0 * u / float(d))"),
    "rope_shift_reversed": ("rope_rotate(Ksel, slots - idx, base, pairing)", "rope_rotate(Ksel, idx - slots, base, pairing)"),
    "rank_lowest_first": ("by_rank = np.argsort(-np.asarray(scores)[idx], kind=\"stable\")",
                          "by_rank = np.argsort(np.asarray(scores)[idx], kind=\"stable\")"),
    "slots_not_inverted": ("slots[by_rank] = np.arange(idx.shape[0], dtype=np.int64)",
                           "slots[:] = by_rank"),
    "values_not_permuted": ("Vout[slots] = Vsel", "Vout[:] = Vsel"),
    "dropped_scale": ("S = (Q @ K.T) / math.sqrt(float(d))", "S = (Q @ K.T)"),
    "scale_by_d": ("/ math.sqrt(float(d))", "/ float(d)"),
    "softmax_wrong_axis": ("mx = S.max(axis=1, keepdims=True)\n    E = np.exp(S - mx)\n    Z = E.sum(axis=1, keepdims=True)",
                           "mx = S.max(axis=0, keepdims=True)\n    E = np.exp(S - mx)\n    Z = E.sum(axis=0, keepdims=True)"),
    "no_normaliser": ("return E / Z", "return E"),
    "sign_of_logits": ("E = np.exp(S - mx)", "E = np.exp(mx - S)"),
    "row_sum_instead_of_column_sum": ("return P.sum(axis=0)", "return P.sum(axis=1)"),
    "mean_instead_of_sum": ("return P.sum(axis=0)", "return P.mean(axis=0)"),
    "chunk_before_cache": ("K = np.concatenate([np.asarray(K_cache), np.asarray(K_chunk)], axis=0)\n    P =",
                           "K = np.concatenate([np.asarray(K_chunk), np.asarray(K_cache)], axis=0)\n    P ="),
    "gather_chunk_before_cache": ("both = np.concatenate([np.asarray(cache), np.asarray(chunk)], axis=0)",
                                  "both = np.concatenate([np.asarray(chunk), np.asarray(cache)], axis=0)"),
    "lowest_scores": ("order = np.argsort(-scores, kind=\"stable\")", "order = np.argsort(scores, kind=\"stable\")"),
    "ties_to_highest_index": ("order = np.argsort(-scores, kind=\"stable\")",
                              "order = (len(scores) - 1 - np.argsort(-scores[::-1], kind=\"stable\"))"),
    "rank_order_output": ("return np.sort(order[:r]).astype(np.int32)", "return order[:r].astype(np.int32)"),
    "off_by_one_r": ("r = max(0, min(int(r), n))", "r = max(0, min(int(r) + 1, n))"),
    "bf16_low_half": ("(x.astype(np.uint32) << np.uint32(16))", "(x.astype(np.uint32))"),
    "values_from_key_rows": ("gather_rows(idx, K_cache, K_chunk), gather_rows(idx, V_cache, V_chunk)",
                             "gather_rows(idx, K_cache, K_chunk), gather_rows(idx, K_cache, K_chunk)"),
    "schedule_ceiling": ("k if constant_budget else (k * seen) // n_cont", "k if constant_budget else -((-k * seen) // n_cont)"),
    "schedule_constant_budget": ("k if constant_budget else (k * seen) // n_cont", "k"),
    "cache_not_carried": ("Kc, Vc = Kn, Vn\n", "Kc, Vc = Kn[:0], Vn[:0]\n"),
    "scores_carried_not_rescored": ("q = Q[i] if isinstance(Q, (list, tuple)) else Q",
                                    "q = Q[0] if isinstance(Q, (list, tuple)) else Q"),
    "positions_not_composed": ("pos = np.concatenate([pos, np.arange(lo, hi, dtype=np.int64)])[idx]",
                               "pos = np.arange(lo, hi, dtype=np.int64)[idx % max(1, hi - lo)]"),
    "reposition_sign": ("return [t - int(old) for t, old in enumerate(ranking)]",
                        "return [int(old) - t for t, old in enumerate(ranking)]"),
}


def load_mutant(old: str, new: str):
    with open(SRC) as f:
        src = f.read()
    assert src.count(old) == 1, f"mutation anchor not found exactly once: {old!r}"
    mod = types.ModuleType("finch_oracle_mutant")
    exec(compile(src.replace(old, new), "finch_oracle_mutant", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_mutation_is_caught(name):
    mod = load_mutant(*MUTATIONS[name])
    failed = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(mod)
        except Exception:                      # any failure counts as "caught"
            failed.append(pin.__name__)
    assert failed, f"mutation {name!r} passed every pin"


def test_unmutated_source_passes():
    with open(SRC) as f:
        src = f.read()
    mod = types.ModuleType("finch_oracle_copy")
    exec(compile(src, "finch_oracle_copy", "exec"), mod.__dict__)
    for pin in oracle_pins.ALL_PINS:
        pin(mod)
