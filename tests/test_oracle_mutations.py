"""Do the pins bite?  Each case plants one plausible mistake in the CPU oracle (a
dropped sign, a wrong shift, a transposed operand, an off-by-one window, a missing
scale, a wrong rounding, a wrong tie-break, ...) and checks that at least one of
the pins of test_oracle_pins.py fails with it.  Everything here runs on the CPU;
the planted mistakes never leave this process."""
import numpy as np
import pytest

from oracle import kvr_oracle as O
import test_oracle_pins as P

MASK64 = (1 << 64) - 1


def fails(pin):
    try:
        pin()
    except Exception:          # an assertion of the pin, or an error the mistake runs into
        return True
    return False


# ---- the planted mistakes: (name, oracle attribute, replacement, pins that should notice) -------------------
def _bucket_low_word(row_params, J, w):
    a, b, _, _ = row_params
    u = (a * J + b) & MASK64
    return ((u & 0xFFFFFFFF) * w) >> 32            # low instead of high 32 bits


def _bucket_no_offset(row_params, J, w):
    a, _, _, _ = row_params
    u = (a * J) & MASK64                           # additive term dropped
    return ((u >> 32) * w) >> 32


def _sign_always_plus(row_params, J):
    return 1


def _sign_from_bucket_params(row_params, J):
    a, b, _, _ = row_params                        # wrong parameter pair
    s = (a * J + b) & MASK64
    return -1 if (s >> 63) else 1


_to_storage = O.to_storage


def _to_storage_truncating(x, storage):
    if storage != "bf16":
        return _to_storage(x, storage)
    x = np.asarray(x)
    if x.dtype == np.float32:
        b = x.copy().view(np.uint32) & np.uint32(0xFFFF0000)
        return b.view(np.float32).astype(np.float64)
    b = x.astype(np.float64).copy().view(np.uint64) & np.uint64(MASK64 ^ ((1 << 45) - 1))
    return b.view(np.float64)


def _to_storage_ties_away(x, storage):
    if storage != "bf16":
        return _to_storage(x, storage)
    x = np.asarray(x)
    if x.dtype == np.float32:
        b = (x.copy().view(np.uint32) + np.uint32(0x8000)) & np.uint32(0xFFFF0000)
        return b.view(np.float32).astype(np.float64)
    b = (x.astype(np.float64).copy().view(np.uint64) + np.uint64(1 << 44)) & np.uint64(MASK64 ^ ((1 << 45) - 1))
    return b.view(np.float64)


_median_rows = O.median_rows


def _median_is_mean(res, median_mode="midmean", storage="f64"):
    return res.mean(axis=1)


def _median_is_max(res, median_mode="midmean", storage="f64"):
    return res.max(axis=1)


def _median_even_upper(res, median_mode="midmean", storage="f64"):
    r = res.shape[1]
    if r % 2 == 1:
        return _median_rows(res, median_mode, storage)
    return np.sort(res, axis=1)[:, r // 2]         # the upper middle value for every rule


_select = O.select


def _select_window_off_by_one(scores, ret_pos, n_ctx, n_recent, k_candidate):
    return _select(scores, ret_pos, n_ctx, n_recent + 1, k_candidate)


def _select_ties_later_first(scores, ret_pos, n_ctx, n_recent, k_candidate):
    recent_from = n_ctx - n_recent
    elig = [s for s in range(len(ret_pos)) if 0 <= ret_pos[s] < recent_from]
    order = sorted(elig, key=lambda s: (-float(scores[ret_pos[s]]), -int(ret_pos[s])))
    keep = set(order[:max(0, k_candidate)])
    ev = [s for s in elig if s not in keep]
    return (np.array(ev, dtype=np.int64), np.array([ret_pos[s] for s in ev], dtype=np.int64))


def _select_lowest_kept(scores, ret_pos, n_ctx, n_recent, k_candidate):
    recent_from = n_ctx - n_recent
    elig = [s for s in range(len(ret_pos)) if 0 <= ret_pos[s] < recent_from]
    order = sorted(elig, key=lambda s: (float(scores[ret_pos[s]]), int(ret_pos[s])))      # ascending: wrong way round
    keep = set(order[:max(0, k_candidate)])
    ev = [s for s in elig if s not in keep]
    return (np.array(ev, dtype=np.int64), np.array([ret_pos[s] for s in ev], dtype=np.int64))


def _attention_without_scale(q, K, V, scale):
    logits = np.asarray(q, dtype=np.float64) @ K.T
    logits = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    p = e / e.sum(axis=1, keepdims=True)
    return p @ V, p


def _attention_unnormalised(q, K, V, scale):
    logits = (np.asarray(q, dtype=np.float64) @ K.T) * scale
    e = np.exp(logits - logits.max(axis=1, keepdims=True))
    return e @ V, e


_insert = O.insert


def _insert_kv_swapped(SK, SV, params, tok_pos, K_tok, V_tok, **kw):
    return _insert(SK, SV, params, tok_pos, V_tok, K_tok, **kw)


def _insert_signs_on_keys(SK, SV, params, tok_pos, K_tok, V_tok, **kw):
    kw = dict(kw)
    kw["sign_mask"] = 1 if kw.get("sign_mask", 2) == 2 else kw["sign_mask"]
    return _insert(SK, SV, params, tok_pos, K_tok, V_tok, **kw)


_query = O.query


def _query_ignores_signs(SK, SV, params, tok_pos, **kw):
    kw = dict(kw)
    kw["sign_mask"] = 0
    return _query(SK, SV, params, tok_pos, **kw)


_swap_pick = O.swap_pick


def _swap_pick_no_rate(scores, ret_pos, vague_pos, n_ctx, n_recent, replace_rate):
    return _swap_pick(scores, ret_pos, vague_pos, n_ctx, n_recent, 1.0)


def _insert_delete_adds(SK, SV, params, tok_pos, K_tok, V_tok, **kw):
    kw = dict(kw)
    if kw.get("coef") is not None:
        kw["coef"] = [abs(int(c)) for c in kw["coef"]]      # V.Delete adds instead of subtracting
    return _insert(SK, SV, params, tok_pos, K_tok, V_tok, **kw)


_revive = O.revive


def _revive_rotated(K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx, **kw):
    K, V = _revive(K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx, **kw)
    vp = [int(p) for p in vague_pos]
    if len(vp) > 1:                                  # every rebuilt token lands on the next Vague position
        K[vp], V[vp] = K[vp[1:] + vp[:1]].copy(), V[vp[1:] + vp[:1]].copy()
    return K, V


_attend_multi = O.attend_multi


def _attend_multi_sees_one_more(q, q_pos, *a, **kw):
    return _attend_multi(q, [int(x) + 1 for x in q_pos], *a, **kw)


HASH = [P.test_bucket_closed_forms, P.test_bucket_range_uniformity_and_sign_balance]
INSERT = [P.test_insert_linearity_and_mass, P.test_insert_sign_mask_variants,
          P.test_insert_rounding_once_per_slot_in_list_order, P.test_whole_step_against_onehot_formulation]
QUERY = [lambda: P.test_query_exact_without_collisions("bf16"), P.test_query_exact_when_majority_of_rows_is_clean,
         P.test_query_single_row_and_brute_force_median, P.test_median_even_rows,
         P.test_whole_step_against_onehot_formulation]
SELECT = [P.test_select_against_lexsort_and_edges, P.test_multi_step_bookkeeping_invariants]
ATTEND = [P.test_attention_matches_library_sdpa, P.test_full_budget_equals_dense_attention_and_score_mass]
SWAP = [P.test_swap_pick_against_brute_force_and_boundaries, P.test_swap_loop_exit_condition_and_partition]
STORAGE = [P.test_to_storage_matches_torch_bf16]
SWAP_BODY = [P.test_swap_restores_token_exactly_without_collisions, P.test_swap_with_collisions_against_onehot_formulation,
             P.test_swap_rounds_shared_slot_once_delete_then_insert]
REVIVE = [P.test_fused_equals_dense_over_reconstruction_and_permutation_invariance,
          P.test_whole_step_against_onehot_formulation]
MULTI = [P.test_attend_multi_against_library_sdpa_with_mask,
         P.test_attend_multi_equals_one_query_at_a_time_on_the_truncated_context]

MUTATIONS = [
    ("bucket from the low word", "bucket_of", _bucket_low_word, HASH),
    ("bucket without the additive term", "bucket_of", _bucket_no_offset, HASH),
    ("sign dropped", "sign_of", _sign_always_plus, HASH + INSERT),
    ("sign from the bucket's parameters", "sign_of", _sign_from_bucket_params, HASH),
    ("storage rounding truncates", "to_storage", _to_storage_truncating, STORAGE),
    ("storage rounding ties away from zero", "to_storage", _to_storage_ties_away, STORAGE),
    ("median replaced by the mean", "median_rows", _median_is_mean, QUERY),
    ("median replaced by the maximum", "median_rows", _median_is_max, QUERY),
    ("even row count: upper middle value", "median_rows", _median_even_upper, QUERY),
    ("Recent window one too long", "select", _select_window_off_by_one, SELECT),
    ("ties: later position ranks higher", "select", _select_ties_later_first, SELECT),
    ("lowest scores kept", "select", _select_lowest_kept, SELECT),
    ("softmax scale missing", "attention", _attention_without_scale, ATTEND),
    ("softmax not normalised", "attention", _attention_unnormalised, ATTEND),
    ("keys and values transposed in the insert", "insert", _insert_kv_swapped, INSERT),
    ("signs on the keys instead of the values", "insert", _insert_signs_on_keys, INSERT),
    ("query ignores the signs", "query", _query_ignores_signs, QUERY + INSERT),
    ("swap decision without ReplaceRate", "swap_pick", _swap_pick_no_rate, SWAP),
    ("delete adds instead of subtracting", "insert", _insert_delete_adds, SWAP_BODY),
    ("rebuilt tokens at the wrong positions", "revive", _revive_rotated, REVIVE),
    ("a query sees one later position", "attend_multi", _attend_multi_sees_one_more, MULTI),
]


def test_pins_pass_unmodified():
    """The reference point: with nothing planted every pin used below passes."""
    for group in (HASH, INSERT, QUERY, SELECT, ATTEND, SWAP, STORAGE, SWAP_BODY, REVIVE, MULTI):
        for pin in group:
            pin()


@pytest.mark.parametrize("name,attr,mutant,pins", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, attr, mutant, pins):
    monkeypatch.setattr(O, attr, mutant)
    caught = [getattr(p, "__name__", "pin") for p in pins if fails(p)]
    assert caught, f"no pin noticed: {name}"


def test_slack_ignored_is_caught(monkeypatch):
    """Algorithm 3's first branch dropped: the Recent part shrinks to its budget after every push."""
    orig = O.UnitState.compress

    def compress_without_slack(self, slack=0):
        return orig(self, 0)

    monkeypatch.setattr(O.UnitState, "compress", compress_without_slack)
    assert fails(lambda: P.test_slack_batches_evictions(3)) or fails(lambda: P.test_slack_against_a_queue_and_a_heap(2))
