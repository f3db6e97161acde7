"""Randomised properties of the CPU oracle (hypothesis): invariants that hold for any
input, on top of the fixed-seed pins of test_oracle_pins.py.  CPU only."""
import math

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import quest_oracle as O
from test_oracle_pins import brute_topk

SETTINGS = dict(max_examples=40, deadline=None)


def _case(seed, B, H, S, D, lens):
    rng = np.random.default_rng(seed)
    pages = [O.num_pages(L, S) for L in lens]
    N = sum(pages) + 1
    ids = rng.permutation(N)
    table = np.zeros((B, max(pages)), np.int32)
    at = 0
    for b in range(B):
        table[b, :pages[b]] = ids[at:at + pages[b]]
        at += pages[b]
    # a coarse grid of values: exact ties and signed zeros are common
    k_pool = (rng.integers(-6, 7, (N, H, S, D)) / 4).astype(np.float16)
    k_pool[rng.random(k_pool.shape) < 0.05] = np.float16(-0.0)
    v_pool = rng.standard_normal((N, H, S, D)).astype(np.float16)
    q = (rng.integers(-8, 9, (B, H, D)) / 4).astype(np.float16)
    return k_pool, v_pool, q, table, np.array(lens, np.int32)


shapes = st.tuples(st.integers(0, 10 ** 6), st.sampled_from([4, 8]), st.sampled_from([4, 8]),
                   st.lists(st.integers(1, 40), min_size=1, max_size=3))


@settings(**SETTINGS)
@given(shapes)
def test_metadata_does_not_depend_on_token_order_and_bounds_every_token(shape):
    seed, S, D, lens = shape
    k_pool, _, _, table, lens = _case(seed, len(lens), 2, S, D, lens)
    meta = O.build_meta(k_pool, table, lens)
    rng = np.random.default_rng(seed + 1)
    shuffled = k_pool.copy()
    for b, L in enumerate(lens):
        for p in range(O.num_pages(L, S)):
            n = O.valid_in_page(L, S, p)
            order = rng.permutation(n)
            shuffled[table[b, p], :, :n] = k_pool[table[b, p], :, :n][:, order]
    again = O.build_meta(shuffled, table, lens)
    assert np.array_equal(meta.view(np.uint16), again.view(np.uint16))          # bit for bit, zeros' signs included
    for b, L in enumerate(lens):
        for p in range(O.num_pages(L, S)):
            n = O.valid_in_page(L, S, p)
            toks = k_pool[table[b, p], :, :n].astype(np.float64)               # [H][n][D]
            assert (meta[:, table[b, p], 0].astype(np.float64)[:, None, :] <= toks).all()
            assert (toks <= meta[:, table[b, p], 1].astype(np.float64)[:, None, :]).all()


@settings(**SETTINGS)
@given(shapes)
def test_score_is_an_upper_bound_reached_by_the_corner_key(shape):
    """Section 3.4: the score bounds q.k for every key inside the page's box, and the key
    that sits in the corner picked by the signs of q reaches it exactly."""
    seed, S, D, lens = shape
    k_pool, _, q, table, lens = _case(seed, len(lens), 2, S, D, lens)
    meta = O.build_meta(k_pool, table, lens)
    sc = O.estimate(meta, q, table, lens, S)
    for b, L in enumerate(lens):
        for p in range(O.num_pages(L, S)):
            n = O.valid_in_page(L, S, p)
            for h in range(2):
                qv = q[b, h].astype(np.float64)
                keys = k_pool[table[b, p], h, :n].astype(np.float64)
                assert sc[b, h, p] >= (keys @ qv).max() - 1e-12
                corner = np.where(qv >= 0, meta[h, table[b, p], 1], meta[h, table[b, p], 0]).astype(np.float64)
                assert math.isclose(sc[b, h, p], float(corner @ qv), rel_tol=1e-13, abs_tol=1e-13)


@settings(**SETTINGS)
@given(st.integers(0, 10 ** 6), st.integers(1, 60), st.integers(1, 70), st.booleans(), st.booleans())
def test_topk_is_repeated_argmax_with_forced_pages_first(seed, P, K, keep_first, keep_newest):
    rng = np.random.default_rng(seed)
    S = 16
    sc = (rng.integers(-5, 6, (1, 1, P + 3)) / 2).astype(np.float64)            # many ties
    sc[0, 0, rng.integers(0, P)] = -0.0
    sc[0, 0, P:] = 1e9                                                          # beyond P: ignored
    lens = np.array([S * (P - 1) + 1 + int(rng.integers(0, S))], np.int32)
    idx, keff = O.topk(sc, lens, S, K, keep_first=keep_first, keep_newest=keep_newest)
    Kb = min(K, P)
    assert keff[0] == Kb and (idx[0, 0, Kb:] == -1).all()
    forced = sorted(set(([0] if keep_first else []) + ([P - 1] if keep_newest else [])))[:Kb]
    rest = [p for p in range(P) if p not in forced]
    fill = brute_topk(sc[0, 0, rest], Kb - len(forced)) if len(forced) < Kb else []
    assert list(idx[0, 0, :Kb]) == sorted(forced + [rest[i] for i in fill])


@settings(**SETTINGS)
@given(shapes, st.integers(1, 6))
def test_attention_over_a_list_is_the_merge_of_attention_over_its_parts(shape, cut):
    """The identity split-K attention rests on: with (o, lse) over two disjoint page sets,
    o = (e^lse_A o_A + e^lse_B o_B) / (e^lse_A + e^lse_B) and lse = log(e^lse_A + e^lse_B)
    are attention over the union; the order of the list does not matter either."""
    seed, S, D, lens = shape
    k_pool, v_pool, q, table, lens = _case(seed, len(lens), 2, S, D, lens)
    B = len(lens)
    maxp = max(O.num_pages(L, S) for L in lens)
    full = np.full((B, 2, maxp), -1, np.int32)
    part_a, part_b = full.copy(), full.copy()
    rng = np.random.default_rng(seed + 2)
    usable = []
    for b, L in enumerate(lens):
        P = O.num_pages(L, S)
        usable.append(P >= 2)
        for h in range(2):
            pages = rng.permutation(P)
            full[b, h, :P] = pages                                              # not sorted on purpose
            c = min(max(1, cut), P - 1) if P >= 2 else P
            part_a[b, h, :c] = np.sort(pages[:c])
            part_b[b, h, :P - c] = np.sort(pages[c:])
    scale = 1 / math.sqrt(D)
    o, lse = O.sparse_decode(k_pool, v_pool, q, table, lens, full, scale)
    dense, dense_lse = O.sparse_decode(k_pool, v_pool, q, table, lens, None, scale)
    assert np.allclose(o, dense, rtol=1e-12, atol=1e-12) and np.allclose(lse, dense_lse, rtol=1e-12)
    for b in range(B):
        if not usable[b]:
            continue
        one = slice(b, b + 1)
        oa, la = O.sparse_decode(k_pool, v_pool, q[one], table[one], lens[one], part_a[one], scale)
        ob, lb = O.sparse_decode(k_pool, v_pool, q[one], table[one], lens[one], part_b[one], scale)
        m = np.maximum(la, lb)
        wa, wb = np.exp(la - m), np.exp(lb - m)
        merged = (wa[..., None] * oa + wb[..., None] * ob) / (wa + wb)[..., None]
        assert np.allclose(merged, o[one], rtol=1e-11, atol=1e-12)
        assert np.allclose(m + np.log(wa + wb), lse[one], rtol=1e-12, atol=1e-12)


@settings(**SETTINGS)
@given(shapes)
def test_appending_token_by_token_is_the_bulk_build(shape):
    seed, S, D, lens = shape
    k_pool, _, _, table, lens = _case(seed, len(lens), 2, S, D, lens)
    start = np.maximum(1, lens // 2).astype(np.int32)
    meta = O.build_meta(k_pool, table, start)
    cur = start.copy()
    while (cur < lens).any():
        grow = cur < lens
        nxt = np.where(grow, cur + 1, cur).astype(np.int32)
        # sequences that do not grow re-fold their last token: folding a key twice changes nothing
        k_new = np.stack([k_pool[table[b, (nxt[b] - 1) // S], :, (nxt[b] - 1) % S] for b in range(len(lens))])
        meta = O.append_meta(meta, k_new, table, nxt, S)
        cur = nxt
    bulk = O.build_meta(k_pool, table, lens)
    for b, L in enumerate(lens):
        ph = table[b, :O.num_pages(L, S)]
        assert np.array_equal(meta[:, ph].view(np.uint16), bulk[:, ph].view(np.uint16))
