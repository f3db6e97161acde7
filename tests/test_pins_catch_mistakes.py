"""The pins are only worth something if a plausible mistake in the oracle fails one of
them.  Each case below plants one mistake in a copy of an oracle function (a dropped
term, a wrong sign or index, a forgotten special case, a different tie rule), swaps it in
for the duration of the test, and checks that the named pin then fails.  CPU only; the
product is never involved."""
import numpy as np
import pytest

import test_oracle_gqa as gqa_pins
import test_oracle_pins as pins
from oracle import quest_oracle as O


# ------------------------------------------------------------------ planted mistakes
def estimate_min_instead_of_max(meta, q, page_table, seq_lens, page_size, max_pages=None):
    sc = O_estimate(meta, q, page_table, seq_lens, page_size, max_pages)
    B, H, D = q.shape
    G = H // meta.shape[0]
    for b in range(B):
        P = O.num_pages(seq_lens[b], page_size)
        sc[b, :, :P] = -np.inf
        for h in range(H):
            qv = q[b, h].astype(np.float64)
            m = meta[h // G, page_table[b, :P], 0].astype(np.float64)
            M = meta[h // G, page_table[b, :P], 1].astype(np.float64)
            sc[b, h // G, :P] = np.maximum(sc[b, h // G, :P], np.minimum(qv * m, qv * M).sum(axis=1))
    return sc


def estimate_drops_last_channel(meta, q, page_table, seq_lens, page_size, max_pages=None):
    q2 = q.copy()
    q2[..., -1] = 0
    return O_estimate(meta, q2, page_table, seq_lens, page_size, max_pages)


def estimate_scaled(meta, q, page_table, seq_lens, page_size, max_pages=None):
    return O_estimate(meta, q, page_table, seq_lens, page_size, max_pages) / np.sqrt(q.shape[-1])


def estimate_uses_max_row_only(meta, q, page_table, seq_lens, page_size, max_pages=None):
    meta2 = meta.copy()
    meta2[:, :, 0] = meta2[:, :, 1]
    return O_estimate(meta2, q, page_table, seq_lens, page_size, max_pages)


def estimate_ignores_page_table(meta, q, page_table, seq_lens, page_size, max_pages=None):
    ident = np.tile(np.arange(page_table.shape[1], dtype=np.int32) % meta.shape[1], (page_table.shape[0], 1))
    sc = O_estimate(meta, q, ident, seq_lens, page_size, max_pages)
    return sc


def topk_higher_page_wins_ties(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    B, H, _ = scores.shape
    idx = np.full((B, H, k_pages), -1, np.int32)
    k_eff = np.zeros(B, np.int32)
    for b in range(B):
        P = O.num_pages(seq_lens[b], page_size)
        K = min(int(k_pages), P)
        k_eff[b] = K
        for h in range(H):
            s = np.asarray(scores[b, h, :P]) + 0.0
            rank = np.lexsort((-np.arange(P), -s))
            idx[b, h, :K] = np.sort(rank[:K])
    return idx, k_eff


def topk_in_rank_order(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    idx, k_eff = O_topk(scores, seq_lens, page_size, k_pages, keep_first, keep_newest)
    for b in range(idx.shape[0]):
        P = O.num_pages(seq_lens[b], page_size)
        for h in range(idx.shape[1]):
            row = idx[b, h, :k_eff[b]]
            idx[b, h, :k_eff[b]] = row[np.argsort(-np.asarray(scores[b, h, :P])[row], kind="stable")]
    return idx, k_eff


def topk_reads_past_the_valid_pages(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    longer = np.asarray(seq_lens) + 2 * page_size
    longer = np.minimum(longer, scores.shape[2] * page_size)
    idx, _ = O_topk(scores, longer, page_size, k_pages, keep_first, keep_newest)
    _, k_eff = O_topk(scores, seq_lens, page_size, k_pages, keep_first, keep_newest)
    return idx, k_eff


def topk_signed_zeros_differ(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    s = np.array(scores, np.float64)
    s = np.where((s == 0) & np.signbit(s), -1e-300, s)
    return O_topk(s, seq_lens, page_size, k_pages, keep_first, keep_newest)


def topk_forced_pages_forgotten(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    return O_topk(scores, seq_lens, page_size, k_pages)


def topk_forced_pages_tie_with_infinite_scores(scores, seq_lens, page_size, k_pages, keep_first=False,
                                               keep_newest=False):
    """Forced pages given the score +inf and ranked like any other score."""
    s = np.array(scores, np.float64)
    for b in range(s.shape[0]):
        P = O.num_pages(seq_lens[b], page_size)
        if keep_first:
            s[b, :, 0] = np.inf
        if keep_newest:
            s[b, :, P - 1] = np.inf
    return O_topk(s, seq_lens, page_size, k_pages)


def build_meta_includes_stale_slots(k_pool, page_table, seq_lens, meta_init=None):
    S = k_pool.shape[2]
    full = np.array([O.num_pages(L, S) * S for L in seq_lens], np.int32)
    return O_build_meta(k_pool, page_table, full, meta_init)


def build_meta_swaps_min_and_max(k_pool, page_table, seq_lens, meta_init=None):
    meta = O_build_meta(k_pool, page_table, seq_lens, meta_init)
    return meta[:, :, ::-1].copy()


def min_without_the_zero_rule(x, axis):
    return x.min(axis=axis)


def append_meta_never_opens_a_page(meta, k_new, page_table, seq_lens, page_size):
    out = meta.copy()
    for b in range(len(seq_lens)):
        pos = int(seq_lens[b]) - 1
        phys = int(page_table[b, pos // page_size])
        k = k_new[b]
        out[:, phys, 0, :] = O._min_total_order(np.stack([out[:, phys, 0, :], k]), axis=0)
        out[:, phys, 1, :] = O._max_total_order(np.stack([out[:, phys, 1, :], k]), axis=0)
    return out


def append_meta_into_the_wrong_page(meta, k_new, page_table, seq_lens, page_size):
    return O_append_meta(meta, k_new, page_table, np.asarray(seq_lens) - 1, page_size)


def decode_ignores_the_scale(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    return O_sparse_decode(k_pool, v_pool, q, page_table, seq_lens, topk_idx, 1.0)


def decode_reads_stale_slots(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    S = k_pool.shape[2]
    full = np.array([O.num_pages(L, S) * S for L in seq_lens], np.int32)
    return O_sparse_decode(k_pool, v_pool, q, page_table, full, topk_idx, sm_scale)


def decode_attends_all_pages(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    return O_sparse_decode(k_pool, v_pool, q, page_table, seq_lens, None, sm_scale)


def decode_swaps_keys_and_values(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    return O_sparse_decode(v_pool, k_pool, q, page_table, seq_lens, topk_idx, sm_scale)


def decode_lse_without_the_max(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    out, lse = O_sparse_decode(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale)
    return out, lse - 1.0


def loaded_fraction_counts_tokens_as_pages(page_size, k_pages, total_pages):
    return 1.0 / page_size + k_pages * page_size / total_pages


O_estimate, O_topk, O_build_meta = O.estimate, O.topk, O.build_meta
O_append_meta, O_sparse_decode = O.append_meta, O.sparse_decode

# (function of the oracle, planted mistake, pin that must fail, its arguments)
CASES = [
    ("estimate", estimate_min_instead_of_max, pins.test_score_upper_bounds_every_token, (0,)),
    ("estimate", estimate_min_instead_of_max, pins.test_score_hand_example, ()),
    ("estimate", estimate_drops_last_channel, pins.test_score_single_token_page_is_the_dot_product, ()),
    ("estimate", estimate_drops_last_channel, pins.test_score_hand_example, ()),
    ("estimate", estimate_scaled, pins.test_score_single_token_page_is_the_dot_product, ()),
    ("estimate", estimate_uses_max_row_only, pins.test_score_sign_definite_queries_and_closed_form, ()),
    ("estimate", estimate_ignores_page_table, pins.test_score_upper_bounds_every_token, (1,)),
    ("estimate", estimate_min_instead_of_max, gqa_pins.test_group_score_bounds_every_logit_of_the_group, ()),
    ("topk", topk_higher_page_wins_ties, pins.test_topk_equals_repeated_argmax, (0,)),
    ("topk", topk_higher_page_wins_ties, pins.test_topk_special_cases, ()),
    ("topk", topk_in_rank_order, pins.test_topk_equals_repeated_argmax, (1,)),
    ("topk", topk_reads_past_the_valid_pages, pins.test_topk_special_cases, ()),
    ("topk", topk_signed_zeros_differ, pins.test_topk_special_cases, ()),
    ("topk", topk_forced_pages_forgotten, pins.test_topk_forced_pages, (True, True)),
    ("topk", topk_forced_pages_tie_with_infinite_scores,
     pins.test_topk_forced_pages_rank_above_infinite_scores, (False, True)),
    ("build_meta", build_meta_includes_stale_slots, pins.test_build_meta_equals_exhaustive_scan, (0,)),
    ("build_meta", build_meta_swaps_min_and_max, pins.test_build_meta_equals_exhaustive_scan, (1,)),
    ("build_meta", build_meta_swaps_min_and_max, pins.test_meta_bounds_every_token_and_ignores_unmapped, ()),
    ("_min_total_order", min_without_the_zero_rule, pins.test_meta_signed_zero_order, ()),
    ("append_meta", append_meta_never_opens_a_page, pins.test_incremental_update_equals_bulk_build, ()),
    ("append_meta", append_meta_into_the_wrong_page, pins.test_incremental_update_equals_bulk_build, ()),
    ("sparse_decode", decode_ignores_the_scale, pins.test_all_pages_selected_is_dense_attention, ()),
    ("sparse_decode", decode_reads_stale_slots, pins.test_all_pages_selected_is_dense_attention, ()),
    ("sparse_decode", decode_attends_all_pages, pins.test_sparse_attention_equals_loops_on_chosen_pages, ()),
    ("sparse_decode", decode_swaps_keys_and_values, pins.test_attention_degenerate_cases, ()),
    ("sparse_decode", decode_lse_without_the_max, pins.test_all_pages_selected_is_dense_attention, ()),
    ("loaded_fraction", loaded_fraction_counts_tokens_as_pages,
     pins.test_loaded_fraction_matches_the_papers_worked_example, ("ROOT",)),
]


@pytest.mark.parametrize("name,mistake,pin,args", CASES,
                         ids=[f"{c[1].__name__}-caught-by-{c[2].__name__}" for c in CASES])
def test_planted_mistake_fails_its_pin(monkeypatch, repo_root, name, mistake, pin, args):
    args = tuple(repo_root if a == "ROOT" else a for a in args)
    pin(*args)                                  # the pin passes on the oracle as it stands
    monkeypatch.setattr(O, name, mistake)
    with pytest.raises(AssertionError):
        pin(*args)
