"""GPU parity of the whole decode step (append -> estimate -> top-k -> sparse
attention) chained on the device, against the oracle chained on the CPU, on the
benchmark configurations: config 0 (tiny) and config 1 at its full size
(32 heads, 32k context, budget 2048) in the launch configuration the benchmark
times, plus the dense (all pages) path on the same buffers."""
import math

import numpy as np
import pytest

from oracle import quest_oracle as O
from paper_2406_10774_amd import synth

pytestmark = pytest.mark.gpu
ATTN_TOL = 2e-3


def torch_index(layer, ids):
    return layer.torch.from_numpy(np.asarray(ids, np.int64)).to(layer.dev)


def run_chain(w, steps, permute, group=1):
    """group > 1: grouped-query attention, w describes the KV heads and every KV head
    serves `group` query heads."""
    import dataclasses
    from gpu_util import Layer, check_selection, score_tolerance
    S, D = w.page_size, w.head_dim
    wq = dataclasses.replace(w, num_heads=w.num_heads * group)    # generator of the queries
    table, N = synth.make_page_table(w, permute=permute)
    k_pool, v_pool, q0 = synth.fill_pools(w, table, N)
    lens = np.array(w.seq_lens, np.int32)
    layer = Layer(k_pool, v_pool, table, lens, num_q_heads=wq.num_heads)
    scale = 1 / math.sqrt(D)

    meta = O.build_meta(k_pool, table, lens)
    got_meta = layer.build_meta()
    mapped = np.unique(np.concatenate([table[b, :w.pages_of(b)] for b in range(w.batch)]))
    assert np.array_equal(got_meta[:, mapped].view(np.uint16), meta[:, mapped].view(np.uint16))

    cur = lens.copy()
    near_ties = 0
    for step in range(steps):
        q = synth.gen_query(wq, step)
        fused = step % 2 == 1                          # odd steps: one launch for append + estimate
        if step > 0:                                   # append one token, then attend
            k_new, v_new = synth.gen_new_token(w, step)
            cur += 1
            layer.set_seq_lens(cur)
            if fused:
                got_sc = layer.append_estimate(k_new, v_new, q)
            else:
                layer.append(k_new, v_new, write=True)
            O.append_kv(k_pool, v_pool, k_new, v_new, table, cur)
            meta = O.append_meta(meta, k_new, table, cur, S)
        sc = O.estimate(meta, q, table, cur, S)
        if not (fused and step > 0):
            got_sc = layer.estimate(q)
        tol = score_tolerance(meta, q, table, cur, S)
        for b in range(w.batch):
            P = -(-int(cur[b]) // S)
            assert (np.abs(got_sc[b, :, :P] - sc[b, :, :P]) <= tol[b, :, :P]).all(), step
        got_idx, keff = layer.topk(w.k_pages)          # from the GPU's own fp32 scores
        near_ties += check_selection(got_idx, sc, cur, S, w.k_pages)
        # attention over the pages the GPU chose, against the oracle on the same pages
        want, want_lse = O.sparse_decode(k_pool, v_pool, q, table, cur, got_idx, scale)
        got, lse = layer.decode(q, got_idx, w.k_pages)
        assert np.abs(got - want).max() <= ATTN_TOL, step
        assert np.abs(lse - want_lse).max() <= ATTN_TOL, step
    # metadata and pools maintained over the steps == oracle's
    got_meta = layer.np16(layer.meta)
    mapped = np.unique(np.concatenate([table[b, :-(-int(cur[b]) // S)] for b in range(w.batch)]))
    assert np.array_equal(got_meta[:, mapped].view(np.uint16), meta[:, mapped].view(np.uint16))
    last = np.array([table[b, (int(cur[b]) - 1) // S] for b in range(w.batch)])
    n_last = [(int(cur[b]) - 1) % S + 1 for b in range(w.batch)]
    got_k, got_v = layer.np16(layer.k_pool[torch_index(layer, last)]), \
        layer.np16(layer.v_pool[torch_index(layer, last)])
    for i, b in enumerate(range(w.batch)):             # the appended tokens landed in their slots
        assert np.array_equal(got_k[i, :, :n_last[b]].view(np.uint16),
                              k_pool[last[b], :, :n_last[b]].view(np.uint16))
        assert np.array_equal(got_v[i, :, :n_last[b]].view(np.uint16),
                              v_pool[last[b], :, :n_last[b]].view(np.uint16))
    # dense path on the same buffers
    q = synth.gen_query(wq, 0)
    want, want_lse = O.sparse_decode(k_pool, v_pool, q, table, cur, None, scale)
    got, lse = layer.decode(q, None, 0)
    assert np.abs(got - want).max() <= ATTN_TOL
    assert np.abs(lse - want_lse).max() <= ATTN_TOL
    return near_ties


def test_config0_chain():
    run_chain(synth.workload(0), steps=5, permute=True)


def test_config1_full_size_chain_identity_table():
    """Same launch configuration as the benchmark (identity page table)."""
    run_chain(synth.workload(1), steps=3, permute=False)


def test_config1_full_size_chain_shuffled_pages():
    run_chain(synth.workload(1), steps=18, permute=True)   # step 17 opens nothing new, 1..16 fill page 2048


def run_decode_steps(w, steps, permute, flags, group=1):
    """quest_decode_step against the separate calls (bit-equal metadata, pools, scores
    and page list) and against the oracle (attention within tolerance).  group > 1:
    grouped-query attention, w describes the KV heads."""
    import dataclasses
    from gpu_util import Layer, check_selection
    S, D = w.page_size, w.head_dim
    wq = dataclasses.replace(w, num_heads=w.num_heads * group)
    table, N = synth.make_page_table(w, permute=permute)
    k_pool, v_pool, _ = synth.fill_pools(w, table, N)
    lens = np.array(w.seq_lens, np.int32)
    meta = O.build_meta(k_pool, table, lens)
    one = Layer(k_pool, v_pool, table, lens, flags=flags, num_q_heads=wq.num_heads)   # one call
    ref = Layer(k_pool, v_pool, table, lens, flags=flags & 12,
                num_q_heads=wq.num_heads)               # separate calls, same selection policy
    one.build_meta()
    ref.build_meta()
    scale = 1 / math.sqrt(D)
    cur = lens.copy()
    for step in range(steps):
        q = synth.gen_query(wq, step)
        k_new, v_new = synth.gen_new_token(w, step)
        append = step % 3 != 2                          # every third step: no new token
        if append:
            cur += 1
            one.set_seq_lens(cur)
            ref.set_seq_lens(cur)
            ref.append(k_new, v_new, write=True)
            O.append_kv(k_pool, v_pool, k_new, v_new, table, cur)
            meta = O.append_meta(meta, k_new, table, cur, S)
        sc1, idx1, keff1, out1, lse1 = one.step(k_new if append else None,
                                                v_new if append else None, q, w.k_pages)
        sc0 = ref.estimate(q)
        idx0, keff0 = ref.topk(w.k_pages)
        for b in range(w.batch):
            P = -(-int(cur[b]) // S)
            assert np.array_equal(sc1[b, :, :P].view(np.uint32), sc0[b, :, :P].view(np.uint32)), step
        assert np.array_equal(idx1, idx0) and np.array_equal(keff1, keff0), step
        if not flags & 12:      # and directly against the selection the oracle's scores imply
            check_selection(idx1, O.estimate(meta, q, table, cur, S), cur, S, w.k_pages)
        if flags & 4:
            assert (idx1[:, :, 0] == 0).all(), step
        if flags & 8:               # the newest page, once: the first page goes before it
            for b in range(w.batch):    # when the list has room for one page only
                newest = (int(cur[b]) - 1) // S
                if keff1[b] >= (2 if flags & 4 and newest != 0 else 1):
                    assert ((idx1[b] == newest).sum(axis=-1) == 1).all(), step
        want, want_lse = O.sparse_decode(k_pool, v_pool, q, table, cur, idx1, scale)
        assert np.abs(out1 - want).max() <= ATTN_TOL, step
        assert np.abs(lse1 - want_lse).max() <= ATTN_TOL, step
    assert np.array_equal(one.np16(one.meta).view(np.uint16), ref.np16(ref.meta).view(np.uint16))
    assert np.array_equal(one.np16(one.k_pool).view(np.uint16), ref.np16(ref.k_pool).view(np.uint16))
    assert np.array_equal(one.np16(one.v_pool).view(np.uint16), ref.np16(ref.v_pool).view(np.uint16))


STEP_FLAGS = [0, 1, 2, 3]   # two launches / three launches / the same two with device fences forced


@pytest.mark.parametrize("flags", STEP_FLAGS)
def test_decode_step_config0(flags):
    run_decode_steps(synth.workload(0), steps=6, permute=True, flags=flags)


@pytest.mark.parametrize("flags", STEP_FLAGS)
def test_decode_step_ragged_batch(flags):
    w = synth.Workload(92, "ragged-step", 5, 3, (1, 16 * 3 + 7, 16 * 203 + 5, 16 * 64, 16 * 130 + 15),
                       token_budget=16 * 24, planted_per_head=4, decode_steps=24)
    run_decode_steps(w, steps=20, permute=True, flags=flags)


@pytest.mark.parametrize("seed", range(24))
def test_decode_step_randomised_shapes(seed):
    """Batch, KV heads, query heads per KV head, page size, sequence lengths, budget and
    flags drawn at random (seeded), a few steps each through quest_decode_step."""
    rng = np.random.default_rng(7000 + seed)
    S = int(rng.choice([8, 16, 32, 64]))
    batch, kv_heads = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    group = int(rng.choice([1, 1, 2, 4]))
    lens = [int(rng.choice([rng.integers(1, 2 * S), rng.integers(2 * S, 40 * S), rng.integers(40 * S, 260 * S)]))
            for _ in range(batch)]
    budget = S * int(rng.choice([1, 2, rng.integers(3, 40), rng.integers(40, 300)]))
    flags = int(rng.choice([0, 1, 2, 3])) | int(rng.choice([0, 0, 4, 8, 12]))
    w = synth.Workload(600 + seed, f"random-{seed}", batch, kv_heads, tuple(lens), token_budget=budget,
                       planted_per_head=4, page_size=S, decode_steps=8)
    print(f"seed {seed}: S={S} batch={batch} kv_heads={kv_heads} group={group} lens={lens} "
          f"budget={budget} flags={flags}", flush=True)
    run_decode_steps(w, steps=5, permute=True, flags=flags, group=group)


@pytest.mark.parametrize("flags", [4 | 8, 1 | 4 | 8, 8])
def test_decode_step_keeps_forced_pages(flags):
    """Selection policy flags through the one-call step (two launches and three launches):
    same list as quest_topk with the same flags; the forced pages are in it."""
    w = synth.Workload(93, "ragged-policy", 4, 3, (1, 16 * 3 + 7, 16 * 203 + 5, 16 * 64),
                       token_budget=16 * 24, planted_per_head=4, decode_steps=24)
    run_decode_steps(w, steps=12, permute=True, flags=flags)


def test_decode_step_long_rows():
    """Rows of ~3000 pages: the selecting attention launch with 8 keys per thread."""
    w = synth.Workload(94, "long-rows-step", 2, 2, (16 * 3000 + 5, 16 * 2600), token_budget=16 * 96,
                       planted_per_head=8, decode_steps=8)
    run_decode_steps(w, steps=5, permute=True, flags=0)


@pytest.mark.parametrize("k_pages", [2048, 2049])
def test_decode_step_at_the_limits_of_the_selecting_launch(k_pages):
    """Rows of 4096 pages and a list of 2048 pages are the largest the attention launch
    selects for itself; one page more in the list and the call is three launches."""
    w = synth.Workload(96, "limits-step", 1, 2, (16 * 4095 + 9,), token_budget=16 * k_pages,
                       planted_per_head=8, decode_steps=4)
    run_decode_steps(w, steps=3, permute=True, flags=0)


@pytest.mark.parametrize("flags", [0, 1])
def test_decode_step_config1_full_size(flags):
    run_decode_steps(synth.workload(1), steps=4, permute=False, flags=flags)
