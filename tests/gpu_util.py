"""Helpers for the GPU parity tests: move a synthetic layer to the device, run
the library through its binding, fetch results back as numpy."""
import math

import numpy as np

from paper_2406_10774_amd import binding as Q


class Layer:
    """Device copy of one layer's paged KV cache plus the buffers of a decode step."""

    def __init__(self, k_pool, v_pool, page_table, seq_lens, meta_fill=None, device="cuda:0",
                 flags=0, num_q_heads=None):
        import torch
        self.torch = torch
        self.dev = device
        N, H, S, D = k_pool.shape
        self.N, self.H, self.S, self.D = N, H, S, D          # H: KV heads
        self.Hq = H if num_q_heads is None else num_q_heads   # query heads (grouped-query attention)
        self.B, self.max_pages = page_table.shape
        self.k_pool = self._to_dev(k_pool)
        self.v_pool = self._to_dev(v_pool)
        self.meta = torch.zeros((H, N, 2, D), dtype=torch.float16, device=device)
        if meta_fill is not None:
            self.meta.fill_(meta_fill)
        self.page_table = torch.from_numpy(np.ascontiguousarray(page_table)).to(device)
        self.seq_lens = torch.from_numpy(np.asarray(seq_lens, np.int32)).to(device)
        self.cache = Q.Cache(self.k_pool, self.v_pool, self.meta, self.page_table, self.seq_lens,
                             flags=flags, num_heads=self.Hq)
        self.scores = torch.full((self.B, H, self.max_pages), float("nan"), dtype=torch.float32,
                                 device=device)

    def _to_dev(self, a):
        t = self.torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(self.dev)
        return t.view(self.torch.float16)

    def half(self, a):
        return self._to_dev(a)

    def set_seq_lens(self, seq_lens):
        self.seq_lens.copy_(self.torch.from_numpy(np.asarray(seq_lens, np.int32)))

    # ---- the five calls
    def build_meta(self):
        Q.quest_build_meta(self.cache)
        return self.np16(self.meta)

    def append(self, k_new, v_new=None, write=False):
        Q.quest_append_meta(self.cache, self.half(k_new), None if v_new is None else self.half(v_new),
                            write)

    def append_estimate(self, k_new, v_new, q, write=True):
        Q.quest_append_estimate(self.cache, self.half(k_new), self.half(v_new), write, self.half(q),
                                self.scores)
        return self.scores.cpu().numpy()

    def estimate(self, q):
        Q.quest_estimate(self.cache, self.half(q), self.scores)
        return self.scores.cpu().numpy()

    def topk(self, k_pages, scores=None):
        torch = self.torch
        if scores is not None:
            self.scores.copy_(torch.from_numpy(np.ascontiguousarray(scores, dtype=np.float32)))
        idx = torch.full((self.B, self.H, k_pages), -7, dtype=torch.int32, device=self.dev)
        keff = torch.full((self.B,), -7, dtype=torch.int32, device=self.dev)
        Q.quest_topk(self.cache, self.scores, k_pages, idx, keff)
        self.idx = idx
        return idx.cpu().numpy(), keff.cpu().numpy()

    def decode(self, q, topk_idx, k_pages, sm_scale=None, fp16_out=False, want_lse=True):
        torch = self.torch
        sm_scale = 1.0 / math.sqrt(self.D) if sm_scale is None else sm_scale
        idx = None
        if topk_idx is not None:
            idx = torch.from_numpy(np.ascontiguousarray(topk_idx, dtype=np.int32)).to(self.dev)
        ws_bytes = Q.quest_workspace_bytes(self.cache, k_pages if idx is not None else 0)
        ws = torch.zeros(max(ws_bytes, 4) // 4, dtype=torch.float32, device=self.dev)
        out = torch.full((self.B, self.Hq, self.D), float("nan"),
                         dtype=torch.float16 if fp16_out else torch.float32, device=self.dev)
        lse = torch.full((self.B, self.Hq), float("nan"), dtype=torch.float32, device=self.dev) \
            if want_lse else None
        Q.quest_sparse_decode(self.cache, self.half(q), idx, k_pages, sm_scale, out, lse, ws)
        torch.cuda.synchronize()
        o = out.cpu().numpy() if not fp16_out else self.np16(out)
        return o, (lse.cpu().numpy() if want_lse else None)

    def select_decode(self, q, k_pages, scores=None, sm_scale=None):
        """Selection and attention in one call, from the scores of the last estimate (or
        the given ones).  Returns (topk_idx, k_eff, out, lse)."""
        torch = self.torch
        sm_scale = 1.0 / math.sqrt(self.D) if sm_scale is None else sm_scale
        sc = self.scores if scores is None else torch.from_numpy(
            np.ascontiguousarray(scores, dtype=np.float32)).to(self.dev)
        ws_bytes = Q.quest_workspace_bytes(self.cache, k_pages)
        ws = torch.zeros(max(ws_bytes, 4) // 4, dtype=torch.float32, device=self.dev)
        idx = torch.full((self.B, self.H, k_pages), -7, dtype=torch.int32, device=self.dev)
        keff = torch.full((self.B,), -7, dtype=torch.int32, device=self.dev)
        out = torch.full((self.B, self.Hq, self.D), float("nan"), dtype=torch.float32, device=self.dev)
        lse = torch.full((self.B, self.Hq), float("nan"), dtype=torch.float32, device=self.dev)
        Q.quest_select_decode(self.cache, self.half(q), sc, k_pages, sm_scale, idx, out, k_eff=keff,
                              lse=lse, workspace=ws)
        torch.cuda.synchronize()
        return idx.cpu().numpy(), keff.cpu().numpy(), out.cpu().numpy(), lse.cpu().numpy()

    def step(self, k_new, v_new, q, k_pages, sm_scale=None, write=True):
        """The whole decode step through the one-call entry point."""
        torch = self.torch
        sm_scale = 1.0 / math.sqrt(self.D) if sm_scale is None else sm_scale
        if getattr(self, "_step_ws_k", None) != k_pages:
            nbytes = Q.quest_step_workspace_bytes(self.cache, k_pages)
            self._step_ws = torch.zeros(max(nbytes, 8) // 4, dtype=torch.int32, device=self.dev)
            self._step_ws_k = k_pages
        idx = torch.full((self.B, self.H, k_pages), -7, dtype=torch.int32, device=self.dev)
        keff = torch.full((self.B,), -7, dtype=torch.int32, device=self.dev)
        out = torch.full((self.B, self.Hq, self.D), float("nan"), dtype=torch.float32, device=self.dev)
        lse = torch.full((self.B, self.Hq), float("nan"), dtype=torch.float32, device=self.dev)
        self.scores.fill_(float("nan"))
        Q.quest_decode_step(self.cache, None if k_new is None else self.half(k_new),
                            None if v_new is None else self.half(v_new), write, self.half(q),
                            k_pages, sm_scale, self.scores, idx, out, self._step_ws, k_eff=keff,
                            lse=lse)
        torch.cuda.synchronize()
        n_counters = min(64 * self.B * self.Hq, self._step_ws.numel())
        assert int(self._step_ws[:n_counters].abs().max().item()) == 0   # counters re-armed
        return (self.scores.cpu().numpy(), idx.cpu().numpy(), keff.cpu().numpy(),
                out.cpu().numpy(), lse.cpu().numpy())

    def np16(self, t):
        return t.view(self.torch.int16).cpu().numpy().view(np.float16)


def score_tolerance(meta, q, page_table, seq_lens, S):
    """fp32 accumulation bound for the criticality score: 128 exact products
    summed in fp32 in any order differ from the exact sum by at most
    (n-1) * 2^-24 * sum|U_i| (n = 128); the DPP tree is far inside that."""
    B, H, D = q.shape
    Hkv = meta.shape[0]
    G = H // Hkv            # query heads per KV head: the group's score is the largest of its
    #                         heads' scores, so its error is at most the largest of their bounds
    tol = np.zeros((B, Hkv, page_table.shape[1]))
    for b in range(B):
        P = -(-int(seq_lens[b]) // S)
        phys = page_table[b, :P]
        for h in range(H):
            qv = q[b, h].astype(np.float64)
            a = np.abs(qv[None] * meta[h // G, phys, 0].astype(np.float64))
            c = np.abs(qv[None] * meta[h // G, phys, 1].astype(np.float64))
            t = np.maximum(a, c).sum(-1) * (D * 2.0 ** -24) + 1e-30
            tol[b, h // G, :P] = np.maximum(tol[b, h // G, :P], t)
    return tol


def check_selection(gpu_idx, oracle_scores, seq_lens, S, k_pages, rel_gap=1e-4):
    """Chained Top-K comparison: GPU selection (from its own fp32 scores) against
    the selection the float64 oracle scores imply.  Where the K-th and (K+1)-th
    oracle scores differ by more than rel_gap (relative), the sets must be equal;
    otherwise pages may differ only among those within rel_gap of the K-th score.
    Returns the number of (b, h) rows that fell under the near-tie rule."""
    B, H, _ = oracle_scores.shape
    near_ties = 0
    for b in range(B):
        P = -(-int(seq_lens[b]) // S)
        K = min(k_pages, P)
        for h in range(H):
            row = gpu_idx[b, h]
            got = row[:K]
            assert (row[K:] == -1).all()
            assert (np.diff(got) > 0).all() and got.min() >= 0 and got.max() < P
            s = oracle_scores[b, h, :P]
            order = np.lexsort((np.arange(P), -s))
            want = np.sort(order[:K])
            if K == P or np.array_equal(got, want):
                continue
            s_k, s_next = s[order[K - 1]], s[order[K]]
            gap = (s_k - s_next) / max(abs(s_k), 1e-30)
            assert gap <= rel_gap, (b, h, gap)
            near_ties += 1
            diff = np.setxor1d(got, want)
            assert (np.abs(s[diff] - s_k) <= rel_gap * max(abs(s_k), 1e-30)).all(), (b, h)
    return near_ties
