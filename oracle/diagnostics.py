"""Selection-quality diagnostics on synthetic data (arXiv 2406.10774, Section 3.2 /
Figure 3 "oracle sparsity" and Figure 4 token recall).

TEST INFRASTRUCTURE ONLY, like the rest of this package: numpy on the host, never
imported by the product.  Nothing here is part of the hot path; it measures how
good a page selection is, with dense attention as the yardstick:

  * attention mass: the share of the dense softmax weight of a (sequence, head)
    that falls on tokens of the selected pages (1 = nothing lost);
  * page recall: how many of the K pages with the largest dense attention mass
    ("oracle" selection, Section 3.2) are in the list;
  * token recall: how many of the n tokens with the largest dense attention
    weight lie in selected pages (the paper's Figure 4 uses n = 10).

The paper's own numbers come from real models and prompts; on the synthetic
keys used here these figures say how the estimate behaves on that distribution,
nothing about model accuracy: "parity unpinned", reported only.

Run as a script for a table:  python -m oracle.diagnostics [--config 0]
"""
from __future__ import annotations

import numpy as np

from . import quest_oracle as O


def attention_weights(k_pool, q_bh, page_table_b, seq_len, h, sm_scale):
    """Dense softmax weights of one (sequence, head) over its seq_len tokens, float64."""
    S, D = k_pool.shape[2], k_pool.shape[3]
    P = O.num_pages(seq_len, S)
    keys = k_pool[page_table_b[:P], h].astype(np.float64).reshape(-1, D)[:int(seq_len)]
    z = sm_scale * (keys @ q_bh.astype(np.float64))
    w = np.exp(z - z.max())
    return w / w.sum()


def selection_quality(k_pool, q, page_table, seq_lens, topk_idx, sm_scale, top_tokens=10):
    """Per (b, h): (attention mass, page recall, token recall) of the lists in topk_idx.
    Returns three float64 arrays [B][H]."""
    B, H, _ = q.shape
    S = k_pool.shape[2]
    mass = np.zeros((B, H))
    page_recall = np.zeros((B, H))
    token_recall = np.zeros((B, H))
    for b in range(B):
        L = int(seq_lens[b])
        P = O.num_pages(L, S)
        for h in range(H):
            w = attention_weights(k_pool, q[b, h], page_table[b], L, h, sm_scale)
            per_page = np.zeros(P)
            np.add.at(per_page, np.arange(L) // S, w)
            row = np.asarray(topk_idx[b, h])
            pages = row[row >= 0]
            chosen = np.zeros(P, bool)
            chosen[pages] = True
            mass[b, h] = per_page[chosen].sum()
            K = len(pages)
            best_pages = np.lexsort((np.arange(P), -per_page))[:K]
            page_recall[b, h] = chosen[best_pages].mean() if K else 1.0
            n = min(top_tokens, L)
            best_tokens = np.lexsort((np.arange(L), -w))[:n]
            token_recall[b, h] = chosen[best_tokens // S].mean()
    return mass, page_recall, token_recall


def report(cid=0, steps=2, heads=None):
    """Quality of Quest's selection on configuration `cid` of the synthetic workloads."""
    from paper_2406_10774_amd import synth
    w = synth.workload(cid)
    if heads is not None:
        import dataclasses
        w = dataclasses.replace(w, num_heads=heads)
    table, N = synth.make_page_table(w, permute=False)
    k_pool, v_pool, _ = synth.fill_pools(w, table, N, stale_fill=0.0)
    lens = np.array(w.seq_lens, np.int32)
    meta = O.build_meta(k_pool, table, lens)
    scale = 1.0 / np.sqrt(w.head_dim)
    rows = []
    for step in range(steps):
        q = synth.gen_query(w, step)
        scores = O.estimate(meta, q, table, lens, w.page_size)
        idx, _ = O.topk(scores, lens, w.page_size, w.k_pages)
        m, pr, tr = selection_quality(k_pool, q, table, lens, idx, scale)
        rows.append((step, m.mean(), m.min(), pr.mean(), tr.mean()))
    return w, rows


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=0)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--heads", type=int, default=None)
    a = ap.parse_args()
    w, rows = report(a.config, a.steps, a.heads)
    print(f"{w.name}: {w.num_heads} heads, {max(w.seq_lens)} tokens, page {w.page_size}, K = {w.k_pages} pages")
    print("query  attention mass (mean / worst head)  page recall  top-10 token recall")
    for step, mm, mw, pr, tr in rows:
        print(f"{step:5d}  {mm:8.4f} / {mw:8.4f}                 {pr:8.4f}     {tr:8.4f}")
