"""fp16 subnormals (|x| < 2^-14) and the largest finite fp16 values (+-65504) in keys,
queries and values, through quest_estimate, quest_sparse_decode and quest_decode_step,
against the oracle.  Products of such operands are exact in fp32 like any other fp16
products, so the usual bars apply; an instruction that flushed subnormal operands to
zero would miss them by far (a subnormal times 65504 is about 4)."""
import math

import numpy as np
import pytest

from oracle import quest_oracle as O
from paper_2406_10774_amd import synth

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def subnormals(rng, shape):
    """Random fp16 subnormals of either sign: m * 2^-24, 1 <= m <= 1023."""
    bits = rng.integers(1, 1024, size=shape).astype(np.uint16) | (rng.integers(0, 2, size=shape).astype(np.uint16) << 15)
    return bits.view(np.float16)


def extremes(rng, shape):
    return (np.where(rng.integers(0, 2, size=shape) == 1, 65504.0, -65504.0)).astype(np.float16)


def salt(arr_k, arr_q, rng):
    """In place: channels 0-7 huge keys x subnormal queries, 8-15 subnormal keys x huge
    queries, 16-23 both subnormal, 24-31 subnormal keys with ordinary queries.  The other
    96 channels keep their ordinary values, so scores and logits stay moderate."""
    arr_k[..., 0:8] = extremes(rng, arr_k[..., 0:8].shape)
    arr_q[..., 0:8] = subnormals(rng, arr_q[..., 0:8].shape)
    arr_k[..., 8:16] = subnormals(rng, arr_k[..., 8:16].shape)
    arr_q[..., 8:16] = extremes(rng, arr_q[..., 8:16].shape)
    arr_k[..., 16:24] = subnormals(rng, arr_k[..., 16:24].shape)
    arr_q[..., 16:24] = subnormals(rng, arr_q[..., 16:24].shape)
    arr_k[..., 24:32] = subnormals(rng, arr_k[..., 24:32].shape)


@pytest.fixture(scope="module")
def salted():
    from gpu_util import Layer
    w = synth.Workload(97, "extreme-values", 3, 4, (16 * 70 + 3, 16 * 9, 5), token_budget=16 * 12,
                       planted_per_head=2, decode_steps=8)
    table, N = synth.make_page_table(w, permute=True)
    k_pool, v_pool, q = synth.fill_pools(w, table, N)
    rng = np.random.default_rng(97)
    q = q.copy()
    salt(k_pool, q, rng)                 # stale slots get values too: they must never be read...
    for b in range(w.batch):             # ...so poison them again
        L, S = int(w.seq_lens[b]), w.page_size
        P = w.pages_of(b)
        if L % S:
            k_pool[table[b, P - 1], :, L % S:] = np.nan
        k_pool[table[b, P:][table[b, P:] >= 0]] = np.nan
    # values: a few subnormal channels (weights < 1 keep the outputs small)
    v_pool[..., 40:48] = np.where(np.isnan(v_pool[..., 40:48]), v_pool[..., 40:48],
                                  subnormals(rng, v_pool[..., 40:48].shape))
    lens = np.array(w.seq_lens, np.int32)
    layer = Layer(k_pool, v_pool, table, lens)
    return w, table, k_pool, v_pool, q, lens, layer


def test_estimate_with_subnormal_and_huge_operands(salted):
    from gpu_util import score_tolerance
    w, table, k_pool, v_pool, q, lens, layer = salted
    meta = O.build_meta(k_pool, table, lens)
    got_meta = layer.build_meta()
    mapped = np.unique(np.concatenate([table[b, :w.pages_of(b)] for b in range(w.batch)]))
    assert np.array_equal(got_meta[:, mapped].view(np.uint16), meta[:, mapped].view(np.uint16))
    want = O.estimate(meta, q, table, lens, w.page_size)
    got = layer.estimate(q)
    tol = score_tolerance(meta, q, table, lens, w.page_size)
    # the salted channels carry weight: without them the scores are off by far more than the bar
    q_plain = q.copy()
    q_plain[..., 0:24] = 0
    without = O.estimate(meta, q_plain, table, lens, w.page_size)
    for b in range(w.batch):
        P = w.pages_of(b)
        assert (np.abs(got[b, :, :P] - want[b, :, :P]) <= tol[b, :, :P]).all(), b
        assert np.abs(without[b, :, :P] - want[b, :, :P]).max() > 100 * tol[b, :, :P].max()


def test_attention_with_subnormal_and_huge_operands(salted):
    w, table, k_pool, v_pool, q, lens, layer = salted
    layer.build_meta()
    scale = 1 / math.sqrt(w.head_dim)
    meta = O.build_meta(k_pool, table, lens)
    sc = O.estimate(meta, q, table, lens, w.page_size)
    idx, _ = O.topk(sc, lens, w.page_size, w.k_pages)
    want, want_lse = O.sparse_decode(k_pool, v_pool, q, table, lens, idx, scale)
    got, lse = layer.decode(q, idx, w.k_pages)
    assert np.abs(got - want).max() <= ATTN_TOL
    assert np.abs(lse - want_lse).max() <= ATTN_TOL
    dense, dense_lse = O.sparse_decode(k_pool, v_pool, q, table, lens, None, scale)
    got, lse = layer.decode(q, None, 0)
    assert np.abs(got - dense).max() <= ATTN_TOL
    assert np.abs(lse - dense_lse).max() <= ATTN_TOL


def test_decode_step_with_subnormal_and_huge_operands(salted):
    from gpu_util import Layer, check_selection
    w, table, k_pool, v_pool, q0, lens, _ = salted
    k_pool, v_pool = k_pool.copy(), v_pool.copy()
    layer = Layer(k_pool, v_pool, table, lens)
    layer.build_meta()
    meta = O.build_meta(k_pool, table, lens)
    scale = 1 / math.sqrt(w.head_dim)
    rng = np.random.default_rng(98)
    cur = lens.copy()
    for step in range(4):
        q = synth.gen_query(w, step)
        k_new, v_new = synth.gen_new_token(w, step)
        salt(k_new, q, rng)
        cur += 1
        layer.set_seq_lens(cur)
        O.append_kv(k_pool, v_pool, k_new, v_new, table, cur)
        meta = O.append_meta(meta, k_new, table, cur, w.page_size)
        sc, idx, keff, out, lse = layer.step(k_new, v_new, q, w.k_pages)
        want_sc = O.estimate(meta, q, table, cur, w.page_size)
        check_selection(idx, want_sc, cur, w.page_size, w.k_pages)
        want, want_lse = O.sparse_decode(k_pool, v_pool, q, table, cur, idx, scale)
        assert np.abs(out - want).max() <= ATTN_TOL, step
        assert np.abs(lse - want_lse).max() <= ATTN_TOL, step
    got_meta = layer.np16(layer.meta)
    mapped = np.unique(np.concatenate([table[b, :-(-int(cur[b]) // w.page_size)] for b in range(w.batch)]))
    assert np.array_equal(got_meta[:, mapped].view(np.uint16), meta[:, mapped].view(np.uint16))


def test_a_single_token_returns_its_value_bit_for_bit():
    """One token in the cache: the softmax weight is exactly 1, so the output is the value
    row itself, also where it holds subnormals and +-65504."""
    from gpu_util import Layer
    w = synth.Workload(99, "one-token", 1, 2, (1,), token_budget=16, planted_per_head=0, decode_steps=1)
    table, N = synth.make_page_table(w, permute=False)
    k_pool, v_pool, q = synth.fill_pools(w, table, N)
    rng = np.random.default_rng(99)
    v_pool[table[0, 0], :, 0, 0:32] = subnormals(rng, (2, 32))
    v_pool[table[0, 0], :, 0, 32:48] = extremes(rng, (2, 16))
    layer = Layer(k_pool, v_pool, table, np.array(w.seq_lens, np.int32))
    idx = np.zeros((1, 2, 1), np.int32)
    got, _ = layer.decode(q, idx, 1)
    want = v_pool[table[0, 0], :, 0].astype(np.float32)[None]
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
