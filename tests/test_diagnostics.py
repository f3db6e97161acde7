"""Pins for the selection-quality diagnostics (oracle/diagnostics.py): closed cases where
attention mass, page recall and token recall are known without computing them the same
way."""
import numpy as np

from oracle import diagnostics as G
from oracle import quest_oracle as O


def tiny(seed=0, P=6, S=4, D=8, H=2):
    rng = np.random.default_rng(seed)
    k_pool = rng.standard_normal((P, H, S, D)).astype(np.float16)
    table = np.arange(P, dtype=np.int32)[None, :]
    lens = np.array([P * S - 1], np.int32)                      # partial last page
    q = rng.standard_normal((1, H, D)).astype(np.float16)
    return k_pool, table, lens, q


def test_everything_selected_loses_nothing():
    k_pool, table, lens, q = tiny()
    idx = np.tile(np.arange(6, dtype=np.int32), (1, 2, 1))
    mass, pr, tr = G.selection_quality(k_pool, q, table, lens, idx, 0.5)
    assert np.allclose(mass, 1.0, atol=1e-12) and (pr == 1).all() and (tr == 1).all()


def test_mass_is_the_sum_of_dense_weights_on_the_chosen_pages():
    k_pool, table, lens, q = tiny(3)
    idx = np.array([[[1, 4, -1], [0, 5, -1]]], np.int32)
    mass, _, _ = G.selection_quality(k_pool, q, table, lens, idx, 0.7)
    for h, pages in enumerate(([1, 4], [0, 5])):
        # explicit loops, Python floats
        z = []
        for t in range(int(lens[0])):
            k = k_pool[t // 4, h, t % 4]
            z.append(0.7 * sum(float(a) * float(b) for a, b in zip(q[0, h], k)))
        m = max(z)
        e = [np.exp(x - m) for x in z]
        want = sum(e[t] for t in range(len(e)) if t // 4 in pages) / sum(e)
        assert abs(mass[0, h] - want) < 1e-12


def test_one_dominant_token():
    """A key equal to a large multiple of q takes almost all the weight: its page alone has
    mass ~1, page recall 1 for K = 1, and any list without it has token recall < 1."""
    k_pool, table, lens, q = tiny(5)
    k_pool[2, 0, 1] = (q[0, 0].astype(np.float32) * 30).astype(np.float16)
    with_it = np.array([[[2], [2]]], np.int32)
    without = np.array([[[3], [3]]], np.int32)
    mass, pr, tr = G.selection_quality(k_pool, q, table, lens, with_it, 1.0, top_tokens=1)
    assert mass[0, 0] > 0.999 and pr[0, 0] == 1 and tr[0, 0] == 1
    mass, pr, tr = G.selection_quality(k_pool, q, table, lens, without, 1.0, top_tokens=1)
    assert mass[0, 0] < 1e-3 and pr[0, 0] == 0 and tr[0, 0] == 0


def test_quest_selection_on_config0_keeps_the_planted_tokens():
    """Config 0 plants 8 tokens with key 3 q0/|q0| (Section 3.4's upper bound guarantees
    their pages score at least 3|q0|); the diagnostics run end to end on it."""
    w, rows = G.report(0, steps=1)
    step, mass_mean, mass_worst, page_recall, token_recall = rows[0]
    assert 0.0 < mass_worst <= mass_mean <= 1.0 + 1e-12
    assert 0.0 <= page_recall <= 1.0 and 0.0 <= token_recall <= 1.0
