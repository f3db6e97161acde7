"""The library's calls captured in a HIP graph: replays (with eager work and
synchronisations between them) give the same results as eager calls.  The library
enqueues kernels only (no memsets, no allocation), so everything is capturable; the
attention launch re-arms its own counters, which is what makes a replay valid."""
import math

import numpy as np
import pytest

from paper_2406_10774_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags", [0, 1])
def test_decode_step_graph_replays_match_eager(flags):
    import torch
    from gpu_util import Layer
    from paper_2406_10774_amd import binding as Q
    w = synth.Workload(95, "graph-small", 3, 4, (16 * 40 + 3, 16 * 130, 16 * 7 + 1),
                       token_budget=16 * 12, planted_per_head=2, decode_steps=16)
    table, N = synth.make_page_table(w, permute=True)
    k_pool, v_pool, _ = synth.fill_pools(w, table, N, stale_fill=0.0)
    lens = np.array(w.seq_lens, np.int32)
    K, D = w.k_pages, w.head_dim
    scale = 1 / math.sqrt(D)

    def fresh():
        layer = Layer(k_pool, v_pool, table, lens + 1, flags=flags)   # the new token is counted
        layer.build_meta()       # over lens + 1: the slot of the new token holds old data, replaced below
        return layer

    q = synth.gen_query(w, 0)
    k_new, v_new = synth.gen_new_token(w, 0)

    def buffers(layer):
        t = layer.torch
        return dict(
            idx=t.full((w.batch, w.num_heads, K), -7, dtype=t.int32, device=layer.dev),
            out=t.zeros((w.batch, w.num_heads, D), dtype=t.float32, device=layer.dev),
            ws=t.zeros(max(Q.quest_step_workspace_bytes(layer.cache, K), 8) // 4, dtype=t.int32,
                       device=layer.dev),
            q=layer.half(q), kn=layer.half(k_new), vn=layer.half(v_new))

    def call(layer, b):
        Q.quest_decode_step(layer.cache, b["kn"], b["vn"], True, b["q"], K, scale, layer.scores,
                            b["idx"], b["out"], b["ws"])

    eager = fresh()
    be = buffers(eager)
    call(eager, be)
    torch.cuda.synchronize()
    want = (eager.scores.clone(), be["idx"].clone(), be["out"].clone(), eager.meta.clone())

    layer = fresh()
    b = buffers(layer)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call(layer, b)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(layer, b)
    for replay in range(4):
        b["idx"].fill_(-7)
        b["out"].zero_()
        layer.scores.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        _ = (b["out"] * 2).sum().item()                  # eager work between replays
        for bb in range(w.batch):
            P = -(-(int(lens[bb]) + 1) // 16)
            assert torch.equal(layer.scores[bb, :, :P].view(torch.int32),
                               want[0][bb, :, :P].view(torch.int32)), replay
        assert torch.equal(b["idx"], want[1]), replay
        assert (b["out"] - want[2]).abs().max().item() <= 1e-5, replay
        assert torch.equal(layer.meta.view(torch.int16), want[3].view(torch.int16)), replay
        n_counters = min(64 * w.batch * w.num_heads, b["ws"].numel())
        assert int(b["ws"][:n_counters].abs().max().item()) == 0     # counters re-armed
