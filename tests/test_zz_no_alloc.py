"""quest_decode_step_static (the decode step with the library's static scratch array
instead of a caller workspace) against quest_decode_step, through the C ABI: two calls
in a row, the second on a smaller input, so that whatever the first call left in the
shared array must not reach the second."""
import math

import numpy as np
import pytest

from paper_2406_10774_amd import synth

pytestmark = pytest.mark.gpu


def _one_step(w, steps=2):
    import torch
    from gpu_util import Layer
    from paper_2406_10774_amd import binding as Q
    table, N = synth.make_page_table(w, permute=True)
    k_pool, v_pool, _ = synth.fill_pools(w, table, N)
    lens = np.array(w.seq_lens, np.int32)
    ref = Layer(k_pool, v_pool, table, lens)
    got = Layer(k_pool, v_pool, table, lens)
    ref.build_meta()
    got.build_meta()
    cur = lens.copy()
    scale = 1 / math.sqrt(w.head_dim)
    for step in range(steps):
        q = synth.gen_query(w, step)
        k_new, v_new = synth.gen_new_token(w, step + 1)
        cur += 1
        ref.set_seq_lens(cur)
        got.set_seq_lens(cur)
        want_sc, want_idx, want_keff, want_out, want_lse = ref.step(k_new, v_new, q, w.k_pages)
        dev = got.dev
        idx = torch.full((got.B, got.H, w.k_pages), -7, dtype=torch.int32, device=dev)
        keff = torch.full((got.B,), -7, dtype=torch.int32, device=dev)
        out = torch.full((got.B, got.Hq, got.D), float("nan"), dtype=torch.float32, device=dev)
        lse = torch.full((got.B, got.Hq), float("nan"), dtype=torch.float32, device=dev)
        got.scores.fill_(float("nan"))
        Q.quest_decode_step_static(got.cache, got.half(k_new), got.half(v_new), True, got.half(q),
                                   w.k_pages, scale, got.scores, idx, out, k_eff=keff, lse=lse)
        torch.cuda.synchronize()
        sc = got.scores.cpu().numpy()
        for b in range(w.batch):
            P = -(-int(cur[b]) // w.page_size)
            assert np.array_equal(sc[b, :, :P].view(np.uint32), want_sc[b, :, :P].view(np.uint32))
        assert np.array_equal(idx.cpu().numpy(), want_idx)          # integer work: bit-exact
        assert np.array_equal(keff.cpu().numpy(), want_keff)
        # same kernels, same split of the list, partial results merged in split order
        assert np.abs(out.cpu().numpy() - want_out).max() <= 2e-3
        assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-3
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want_out.view(np.uint32))
    same = lambda a, b: bool(torch.equal(a.view(torch.int16), b.view(torch.int16)))  # stale slots are NaN
    assert same(got.meta, ref.meta), "metadata"
    assert same(got.k_pool, ref.k_pool) and same(got.v_pool, ref.v_pool), "pools"


def test_static_scratch_matches_workspace_on_two_calls_in_a_row():
    big = synth.Workload(71, "static-big", 3, 8, (16 * 300 - 5, 16 * 120 + 1, 700), 16 * 40, 4,
                         decode_steps=4)
    small = synth.Workload(72, "static-small", 1, 4, (16 * 90 + 7,), 16 * 24, 2, decode_steps=4)
    _one_step(big)
    _one_step(small)


def test_static_scratch_refuses_shapes_beyond_its_size():
    import torch
    from paper_2406_10774_amd import binding as Q
    dev = "cuda:0"
    B, H, P = 16, 32, 32768                      # 8 chunks x 512 candidates per row: 16 MiB of scratch
    pools = torch.zeros((1, H, 16, 128), dtype=torch.float16, device=dev)
    meta = torch.zeros((H, 1, 2, 128), dtype=torch.float16, device=dev)
    pt = torch.zeros((B, P), dtype=torch.int32, device=dev)
    lens = torch.full((B,), 16 * P, dtype=torch.int32, device=dev)
    cache = Q.Cache(pools, pools, meta, pt, lens)
    assert Q.quest_step_workspace_bytes(cache, 512) > 4 << 20
    q = torch.zeros((B, H, 128), dtype=torch.float16, device=dev)
    scores = torch.zeros((B, H, P), dtype=torch.float32, device=dev)
    idx = torch.zeros((B, H, 512), dtype=torch.int32, device=dev)
    out = torch.zeros((B, H, 128), dtype=torch.float32, device=dev)
    with pytest.raises(Q.QuestError) as err:
        Q.quest_decode_step_static(cache, None, None, False, q, 512, 0.1, scores, idx, out)
    assert err.value.status == -4
