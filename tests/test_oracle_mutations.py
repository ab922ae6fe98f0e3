"""Mutation checks of the pins: every planted mistake below (a dropped term, a
wrong sign or index, a transposed operand, a wrong tie-break) is patched into the
CPU oracle, and at least one pin of tests/test_oracle_pins.py has to fail.  A
mistake that survives means the pins do not constrain that part of the oracle.
Everything here runs on the CPU; nothing is planted in the GPU path."""
import numpy as np
import pytest

from oracle import hack_oracle as ho
from tests import test_oracle_pins as pins


def _run_pins():
    """Run every pin (parametrised ones with their parameters); return the names that failed."""
    failed = []

    def call(name, fn, *args):
        try:
            fn(*args)
        except AssertionError:
            failed.append(name)
        except Exception as e:  # a mutant may also break shapes: that counts as caught
            failed.append(f"{name} ({type(e).__name__})")

    call("observation_rows", pins.test_observation_rows_stride_and_small_scales)
    for p in [(3, 7, 4, 0.5), (5, 11, 6, 0.37), (1, 4, 3, 1.0)]:
        call("importance_pure_python", pins.test_importance_matches_pure_python, *p)
    call("importance_closed_forms", pins.test_importance_closed_forms)
    call("importance_invariants", pins.test_importance_invariants_and_scale)
    call("topk_hand", pins.test_topk_hand_computed)
    call("structural_hand", pins.test_structural_hand_computed)
    call("structural_small_budget", pins.test_structural_small_budget_reading)
    call("all_equal", pins.test_all_equal_importance_closed_form)
    call("float32_decision", pins.test_decision_is_taken_in_float32)
    for seed in range(6):
        call("select_brute_force", pins.test_select_matches_brute_force_and_invariants, seed)
    call("compact", pins.test_compact_is_a_row_gather)
    call("attention", pins.test_attention_matches_pure_python_and_properties)
    call("full_budget_schedule", pins.test_full_budget_schedule_is_vanilla_cache_attention)
    call("budget_equal", pins.test_budget_equal_to_cache_is_not_compressed_and_budget_100_equals_full)
    call("compress_before_attention", pins.test_unit_step_compresses_before_attention)
    call("schedule_invariants", pins.test_schedule_invariants_under_compression)
    for prm in [(4, 9, 5, 0.6), (7, 3, 4, 1.3), (2, 6, 3, 0.25)]:
        call("head_variance_pure_python", pins.test_head_variance_matches_pure_python, *prm)
    call("head_variance_closed_forms", pins.test_head_variance_closed_forms_and_invariants)
    call("classify_heads", pins.test_classify_heads_hand_computed_and_planted_mask)
    for prm in [(0, 9, 4, 5), (1, 14, 3, 8), (2, 6, 5, 3), (3, 12, 1, 4)]:
        call("merge_pure_python", pins.test_merge_matches_pure_python, *prm)
    call("merge_hand", pins.test_merge_hand_computed_four_keys)
    call("merge_properties", pins.test_merge_properties)
    call("merge_final_step_only", pins.test_merge_happens_only_for_contextual_heads_at_the_final_step)
    return failed


def test_the_unmutated_oracle_passes_every_pin():
    assert _run_pins() == []


# ---- planted mistakes -------------------------------------------------------
def _softmax_no_normaliser(S):
    S = S - S.max(axis=1, keepdims=True)
    return np.exp(S)


def _softmax_over_queries(S):                     # normalises the wrong axis
    S = S - S.max(axis=0, keepdims=True)
    E = np.exp(S)
    return E / E.sum(axis=0, keepdims=True)


def _subset_attention_no_scale(Q_obs, K, scale):
    return ho.softmax_rows(Q_obs @ K.T)


def _subset_attention_negated(Q_obs, K, scale):
    return ho.softmax_rows(-scale * (Q_obs @ K.T))


def _importance_mean_instead_of_sum(Q_obs, K, scale):
    return ho.subset_attention(Q_obs, K, scale).mean(axis=0)


def _importance_max_instead_of_sum(Q_obs, K, scale):
    return ho.subset_attention(Q_obs, K, scale).max(axis=0)


def _observation_rows_first_rows(N_k, N_obs=32):  # first rows instead of a strided sample
    return np.arange(min(N_obs, N_k), dtype=np.int64)


def _observation_rows_ceil(N_k, N_obs=32):
    n_obs = min(N_obs, N_k)
    i = np.arange(n_obs, dtype=np.int64)
    return np.minimum(-((-i * N_k) // n_obs) + (N_k > n_obs), N_k - 1)


def _topk_smallest(values, k):
    return _orig_topk(-values, k)


def _topk_ties_to_higher_index(values, k):
    k = int(k)
    n = values.shape[0]
    if k <= 0:
        return np.zeros(0, np.int64)
    if k >= n:
        return np.arange(n, dtype=np.int64)
    order = np.argsort(-values[::-1], kind="stable")
    return np.sort((n - 1 - order)[:k]).astype(np.int64)


def _topk_unsorted_output(values, k):
    k = int(k)
    n = values.shape[0]
    if k <= 0:
        return np.zeros(0, np.int64)
    if k >= n:
        return np.arange(n, dtype=np.int64)
    return np.argsort(-values, kind="stable")[:k].astype(np.int64)


def _topk_one_short(values, k):
    return _orig_topk(values, max(int(k) - 1, 0))


def _structural_no_init(imp, B_S, N_init, N_k):
    return _orig_structural(imp, B_S, 0, N_k)


def _structural_recent_off_by_one(imp, B_S, N_init, N_k):
    return _orig_structural(imp, B_S, N_init, max(int(N_k) - 1, 0))


def _structural_ranks_whole_cache(imp, B_S, N_init, N_k):   # forgets the protected windows
    return ho.select_contextual(imp, B_S)


def _structural_decides_in_float64(imp, B_S, N_init, N_k):
    saved = ho.decision_values
    ho.decision_values = lambda x: np.asarray(x, dtype=np.float64)
    try:
        return _orig_structural(imp, B_S, N_init, N_k)
    finally:
        ho.decision_values = saved


def _contextual_decides_in_float64(imp, B_C):
    return ho.topk_indices(np.asarray(imp, np.float64), min(int(B_C), imp.shape[0]))


def _compact_swaps_k_and_v(K, V, I):
    return V[I], K[I]


def _compact_reversed(K, V, I):
    return K[I[::-1]], V[I[::-1]]


def _attention_transposed_scores(Q, K, V, scale):
    S = scale * (Q @ K.T)
    P = _softmax_over_queries(S)
    return P @ V


def _attention_no_scale(Q, K, V, scale):
    return ho.softmax_rows(Q @ K.T) @ V


def _attention_uses_keys_as_values(Q, K, V, scale):
    return ho.softmax_rows(scale * (Q @ K.T)) @ K


def _attention_causal(Q, K, V, scale):               # a mask inside the scale step
    S = scale * (Q @ K.T)
    n_q, n_k = S.shape
    j = np.arange(n_k)[None, :]
    i = np.arange(n_q)[:, None] + (n_k - n_q)
    return ho.softmax_rows(np.where(j <= i, S, -1e30)) @ V


def _variance_sample_instead_of_population(Q, K, scale):
    A = ho.softmax_rows(scale * (Q @ K.T))
    return float(A.var(axis=0, ddof=1).sum())


def _variance_across_keys(Q, K, scale):              # row-wise instead of column-wise
    A = ho.softmax_rows(scale * (Q @ K.T))
    return float(A.var(axis=1).sum())


def _variance_of_logits(Q, K, scale):                # forgets the softmax
    return float((scale * (Q @ K.T)).var(axis=0).sum())


def _variance_mean_over_columns(Q, K, scale):
    A = ho.softmax_rows(scale * (Q @ K.T))
    return float(A.var(axis=0).mean())


def _classify_high_variance_is_contextual(sigma, alpha):
    return _orig_classify(-np.asarray(sigma, np.float64), alpha)


def _classify_per_layer_ranking(sigma, alpha):       # ranks inside each layer instead of globally
    sigma = np.asarray(sigma, np.float64)
    if sigma.ndim < 2:
        return _orig_classify(sigma, alpha)
    return np.stack([_orig_classify(row, alpha) for row in sigma])


_orig_topk = ho.topk_indices
_orig_classify = ho.classify_heads
_orig_structural = ho.select_structural

def _merge_with(sim=None, pick=np.argmax, clip=True, own_weight=1.0, v_uniform=False):
    """merge_final rebuilt from its steps with one of them replaced."""
    def merge(K, V, I):
        T = K.shape[0]
        I = np.asarray(I, dtype=np.int64)
        ev = np.setdiff1d(np.arange(T, dtype=np.int64), I)
        Kh, Vh = K[I].copy(), V[I].copy()
        if ev.size == 0:
            return Kh, Vh, np.zeros(0, np.int64), np.zeros(0)
        S = (sim or ho.key_similarity)(K[ev], K[I])
        nearest = pick(S, axis=1)
        w = S[np.arange(ev.size), nearest]
        if clip:
            w = np.maximum(w, 0.0)
        tot = np.full(I.size, own_weight)
        Kh, Vh = Kh * own_weight, Vh * own_weight
        np.add.at(Kh, nearest, w[:, None] * K[ev])
        np.add.at(Vh, nearest, (np.ones_like(w) if v_uniform else w)[:, None] * V[ev])
        np.add.at(tot, nearest, w)
        return Kh / tot[:, None], Vh / tot[:, None], nearest.astype(np.int64), w
    return merge


def _merge_farthest(K, V, I):
    return _merge_with(pick=np.argmin)(K, V, I)


def _merge_plain_dot_similarity(K, V, I):
    return _merge_with(sim=lambda A, B: A @ B.T)(K, V, I)


def _merge_negative_weights_kept(K, V, I):
    return _merge_with(clip=False)(K, V, I)


def _merge_kept_row_without_own_weight(K, V, I):
    return _merge_with(own_weight=1e-9)(K, V, I)


def _merge_values_unweighted(K, V, I):
    return _merge_with(v_uniform=True)(K, V, I)


def _merge_is_a_plain_gather(K, V, I):            # the merge forgotten
    I = np.asarray(I, dtype=np.int64)
    return K[I], V[I], np.zeros(0, np.int64), np.zeros(0)


def _merge_ties_to_higher_index(K, V, I):
    return _merge_with(pick=lambda S, axis: S.shape[1] - 1 - np.argmax(S[:, ::-1], axis=axis))(K, V, I)


def _similarity_unnormalised_by_one_side(K_a, K_b):
    nb = np.sqrt((K_b * K_b).sum(axis=1))
    return (K_a @ K_b.T) / nb[None, :]


MUTANTS = [
    ("softmax_rows", _softmax_no_normaliser),
    ("softmax_rows", _softmax_over_queries),
    ("subset_attention", _subset_attention_no_scale),
    ("subset_attention", _subset_attention_negated),
    ("importance", _importance_mean_instead_of_sum),
    ("importance", _importance_max_instead_of_sum),
    ("observation_rows", _observation_rows_first_rows),
    ("observation_rows", _observation_rows_ceil),
    ("topk_indices", _topk_smallest),
    ("topk_indices", _topk_ties_to_higher_index),
    ("topk_indices", _topk_unsorted_output),
    ("topk_indices", _topk_one_short),
    ("select_structural", _structural_no_init),
    ("select_structural", _structural_recent_off_by_one),
    ("select_structural", _structural_ranks_whole_cache),
    ("select_structural", _structural_decides_in_float64),
    ("select_contextual", _contextual_decides_in_float64),
    ("compact", _compact_swaps_k_and_v),
    ("compact", _compact_reversed),
    ("attention", _attention_transposed_scores),
    ("attention", _attention_no_scale),
    ("attention", _attention_uses_keys_as_values),
    ("attention", _attention_causal),
    ("head_variance", _variance_sample_instead_of_population),
    ("head_variance", _variance_across_keys),
    ("head_variance", _variance_of_logits),
    ("head_variance", _variance_mean_over_columns),
    ("classify_heads", _classify_high_variance_is_contextual),
    ("classify_heads", _classify_per_layer_ranking),
    ("merge_final", _merge_farthest),
    ("merge_final", _merge_plain_dot_similarity),
    ("merge_final", _merge_negative_weights_kept),
    ("merge_final", _merge_kept_row_without_own_weight),
    ("merge_final", _merge_values_unweighted),
    ("merge_final", _merge_is_a_plain_gather),
    ("merge_final", _merge_ties_to_higher_index),
    ("key_similarity", _similarity_unnormalised_by_one_side),
]


@pytest.mark.parametrize("target,mutant", MUTANTS, ids=[f"{t}:{m.__name__.lstrip('_')}" for t, m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, target, mutant):
    monkeypatch.setattr(ho, target, mutant)
    failed = _run_pins()
    assert failed, f"no pin noticed {mutant.__name__} planted into oracle.{target}"


def test_merge_at_the_wrong_place_is_caught(monkeypatch):
    """A schedule that merges for structural heads too, or at every step."""
    orig = ho.unit_step

    def merge_everywhere(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw):
        kw = dict(kw)
        if "final_merge" in kw or len(a) >= 3:
            kw["final_merge"] = True
            a = a[:2]
        return orig(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw)

    def merge_structural(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw):
        r = dict(orig(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw))
        if kw.get("final_merge") and head_type == ho.STRUCTURAL and r["compressed"]:
            K_in, V_in = np.concatenate([Kc, Kk]), np.concatenate([Vc, Vk])
            r["K"], r["V"], _, _ = ho.merge_final(K_in, V_in, r["I"])
            r["O"] = ho.attention(Qk, r["K"], r["V"], scale)
        return r

    for planted in (merge_everywhere, merge_structural):
        monkeypatch.setattr(ho, "unit_step", planted)
        failed = _run_pins()
        assert "merge_final_step_only" in failed, (planted.__name__, failed)


def test_compress_after_attention_is_caught(monkeypatch):
    """A schedule that attends over the uncompressed keys and compresses afterwards."""
    orig = ho.unit_step

    def late(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw):
        out = dict(orig(Kc, Vc, Pc, Qk, Kk, Vk, pos0, head_type, budget, N_init, scale, *a, **kw))
        out["O"] = ho.attention(Qk, np.concatenate([Kc, Kk]), np.concatenate([Vc, Vk]), scale)
        return out

    monkeypatch.setattr(ho, "unit_step", late)
    failed = _run_pins()
    assert any(name.startswith("compress_before_attention") or name.startswith("schedule_invariants")
               for name in failed), failed
