"""Pins for the grouped-query reading of the oracle (fewer KV heads than query heads):
it must equal the one-KV-head-per-query-head path (pinned in test_oracle_pins.py) on the
same problem with every KV head repeated G times, with the group's page score the largest
of its heads' scores; and the group score must bound every logit of every head of the
group (the property that makes it a criticality estimate, Section 3.4), by explicit loops."""
import numpy as np

from oracle import quest_oracle as O


def problem(seed=0, B=2, Hkv=2, G=3, S=8, D=16, P=7):
    rng = np.random.default_rng(seed)
    N = B * P
    k_pool = rng.standard_normal((N, Hkv, S, D)).astype(np.float16)
    v_pool = rng.standard_normal((N, Hkv, S, D)).astype(np.float16)
    table = rng.permutation(N).astype(np.int32).reshape(B, P)
    lens = np.array([P * S - 3, 2 * S + 1], np.int32)[:B]
    q = rng.standard_normal((B, Hkv * G, D)).astype(np.float16)
    return k_pool, v_pool, table, lens, q, G


def test_group_score_is_the_max_of_its_heads_scores_on_repeated_kv():
    k_pool, v_pool, table, lens, q, G = problem()
    S = k_pool.shape[2]
    meta = O.build_meta(k_pool, table, lens)
    got = O.estimate(meta, q, table, lens, S)                          # [B][Hkv][P]
    wide = O.estimate(np.repeat(meta, G, axis=0), q, table, lens, S)   # [B][H][P], one KV head each
    want = wide.reshape(wide.shape[0], -1, G, wide.shape[2]).max(axis=2)
    assert np.array_equal(got, want)


def test_group_score_bounds_every_logit_of_the_group():
    k_pool, v_pool, table, lens, q, G = problem(1)
    S = k_pool.shape[2]
    meta = O.build_meta(k_pool, table, lens)
    sc = O.estimate(meta, q, table, lens, S)
    for b in range(q.shape[0]):
        for h in range(q.shape[1]):
            for p in range(O.num_pages(lens[b], S)):
                for s_ in range(O.valid_in_page(lens[b], S, p)):
                    k = k_pool[table[b, p], h // G, s_]
                    logit = sum(float(a) * float(c) for a, c in zip(q[b, h], k))
                    assert sc[b, h // G, p] >= logit - 1e-9


def test_attention_with_a_shared_list_equals_repeated_kv():
    k_pool, v_pool, table, lens, q, G = problem(2)
    S = k_pool.shape[2]
    meta = O.build_meta(k_pool, table, lens)
    sc = O.estimate(meta, q, table, lens, S)
    idx, keff = O.topk(sc, lens, S, 3)                                 # [B][Hkv][3]
    out, lse = O.sparse_decode(k_pool, v_pool, q, table, lens, idx, 0.3)
    wide_out, wide_lse = O.sparse_decode(np.repeat(k_pool, G, axis=1), np.repeat(v_pool, G, axis=1), q,
                                         table, lens, np.repeat(idx, G, axis=1), 0.3)
    assert np.array_equal(out, wide_out) and np.array_equal(lse, wide_lse)
    dense, _ = O.sparse_decode(k_pool, v_pool, q, table, lens, None, 0.3)
    wide_dense, _ = O.sparse_decode(np.repeat(k_pool, G, axis=1), np.repeat(v_pool, G, axis=1), q,
                                    table, lens, None, 0.3)
    assert np.array_equal(dense, wide_dense)
