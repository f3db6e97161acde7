"""CPU oracle for the Quest decode hot path (arXiv 2406.10774).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
statement of what the hot path computes, written from the paper.  It shares no
code with the HIP kernels and must never be imported by the product package:
only tests, the smoke check and the benchmark's CPU-baseline leg call it.

Everything is numpy on the host.  Order comparisons (min/max metadata, Top-K)
are exact; floating-point steps (criticality score, attention) convert the
fp16 inputs to float64 and accumulate in float64.

Shapes (C order):
  k_pool, v_pool : float16 [N][H][S][D]    N physical pages, S tokens per page
  meta           : float16 [H][N][2][D]    [..,0,:] = channel-wise min, [..,1,:] = max
  page_table     : int32   [B][max_pages]  logical page p of sequence b -> physical page
  seq_lens       : int32   [B]             valid tokens; logical page p holds tokens [pS, pS+S)
  q              : float16 [B][H][D]
  scores         : float64 [B][H][max_pages]  (entries p >= P_b are -inf)
  topk_idx       : int32   [B][H][K]       ascending logical page ids, padded with -1

Readings of points the paper leaves open (each also applies to the HIP path):
  * A page's metadata starts from its first token (m = M = k); Algorithm 1 only
    gives the update rule.
  * min/max use the total order "by value, and -0 below +0", so the result does
    not depend on the order tokens are folded in.  NaN keys are excluded.
  * A partial last page contributes only its valid tokens, to metadata and to
    attention alike.
  * Selection is independent per (sequence, head); scores are unscaled
    (Algorithm 1 has no 1/sqrt(d)).
  * Top-K: K = min(k_pages, P_b); equal scores are resolved towards the lower
    page index; the chosen pages are reported in ascending page order.
  * The softmax scale is an argument (tests use 1/sqrt(D)).

Pins (tests/test_oracle_*.py): exhaustive per-token scans, the upper-bound
property of Section 3.4, the single-token and sign-definite special cases, the
closed form 1/2 sum[q(M+m) + |q|(M-m)], selection by repeated arg-max, dense
attention written as explicit loops, logsumexp from scipy.  The one thing with
no pin is how close sparse attention is to dense attention: the paper gives no
error bound for it, so that distance is "parity unpinned" and only reported.
"""
from __future__ import annotations

import numpy as np


def num_pages(seq_len: int, page_size: int) -> int:
    """P = ceil(L / S) logical pages hold L tokens."""
    return -(-int(seq_len) // int(page_size))


def valid_in_page(seq_len: int, page_size: int, p: int) -> int:
    """Number of valid tokens in logical page p (S, except a partial last page)."""
    return int(min(page_size, int(seq_len) - p * page_size))


# --------------------------------------------------------------------------
# Section 3.4 / Algorithm 1 (insertion half): per-page channel-wise min and max
# --------------------------------------------------------------------------

def _min_total_order(x: np.ndarray, axis: int) -> np.ndarray:
    """Minimum along `axis` under 'by value, -0 < +0'."""
    v = x.min(axis=axis)
    neg_zero_present = ((x == 0) & np.signbit(x)).any(axis=axis)
    is_zero = (v == 0)
    out = v.copy()
    out[is_zero & neg_zero_present] = np.float16(-0.0)
    out[is_zero & ~neg_zero_present] = np.float16(0.0)
    return out


def _max_total_order(x: np.ndarray, axis: int) -> np.ndarray:
    """Maximum along `axis` under 'by value, -0 < +0'."""
    v = x.max(axis=axis)
    pos_zero_present = ((x == 0) & ~np.signbit(x)).any(axis=axis)
    is_zero = (v == 0)
    out = v.copy()
    out[is_zero & pos_zero_present] = np.float16(0.0)
    out[is_zero & ~pos_zero_present] = np.float16(-0.0)
    return out


def build_meta(k_pool, page_table, seq_lens, meta_init=None):
    """Metadata of every mapped page: m_i = min_j k_{j,i}, M_i = max_j k_{j,i}
    over the valid tokens j of the page (Section 3.4).

    Returns meta float16 [H][N][2][D]; entries of pages that hold no valid
    token keep the value of `meta_init` (zeros if not given)."""
    N, H, S, D = k_pool.shape
    meta = np.zeros((H, N, 2, D), np.float16) if meta_init is None else meta_init.copy()
    for b in range(len(seq_lens)):
        L = int(seq_lens[b])
        P = num_pages(L, S)
        for p in range(P):
            n = valid_in_page(L, S, p)
            phys = int(page_table[b, p])
            toks = k_pool[phys, :, :n, :]                 # [H][n][D]
            meta[:, phys, 0, :] = _min_total_order(toks, axis=1)
            meta[:, phys, 1, :] = _max_total_order(toks, axis=1)
    return meta


def append_meta(meta, k_new, page_table, seq_lens, page_size):
    """Fold the newest token's key into its page (Algorithm 1, insertion half).

    seq_lens already counts the new token: it sits at position L-1, i.e. slot
    (L-1) mod S of logical page (L-1) div S.  Slot 0 opens the page: m = M = k.
    Otherwise M = max(M, k), m = min(m, k).  Returns the updated copy."""
    out = meta.copy()
    for b in range(len(seq_lens)):
        pos = int(seq_lens[b]) - 1
        phys = int(page_table[b, pos // page_size])
        k = k_new[b]                                        # [H][D]
        if pos % page_size == 0:
            out[:, phys, 0, :] = k
            out[:, phys, 1, :] = k
        else:
            out[:, phys, 0, :] = _min_total_order(np.stack([out[:, phys, 0, :], k]), axis=0)
            out[:, phys, 1, :] = _max_total_order(np.stack([out[:, phys, 1, :], k]), axis=0)
    return out


def append_kv(k_pool, v_pool, k_new, v_new, page_table, seq_lens):
    """Store the newest token's key and value in its slot (in place)."""
    S = k_pool.shape[2]
    for b in range(len(seq_lens)):
        pos = int(seq_lens[b]) - 1
        phys = int(page_table[b, pos // S])
        k_pool[phys, :, pos % S, :] = k_new[b]
        v_pool[phys, :, pos % S, :] = v_new[b]


# --------------------------------------------------------------------------
# Section 3.4 / Algorithm 1 (attention half): criticality score per page
# --------------------------------------------------------------------------

def estimate(meta, q, page_table, seq_lens, page_size, max_pages=None):
    """score[b,h,p] = sum_i max(q_i * m_{p,i}, q_i * M_{p,i}), unscaled, float64.

    Entries p >= P_b are -inf.

    Grouped-query attention (the paper's models have one KV head per query head
    and it gives no rule for groups; this is the reading used here): when meta
    has fewer heads than q, query heads [g*G, (g+1)*G) share KV head g, each
    query head is scored against that head's metadata, and the score of the page
    for the group is the largest of its heads' scores: still an upper bound of
    every logit any head of the group can reach in the page.  One row per KV
    head is returned."""
    B, H, D = q.shape
    Hkv = meta.shape[0]
    G = H // Hkv
    assert G * Hkv == H
    max_pages = page_table.shape[1] if max_pages is None else max_pages
    scores = np.full((B, Hkv, max_pages), -np.inf, np.float64)
    for b in range(B):
        P = num_pages(seq_lens[b], page_size)
        phys = page_table[b, :P]
        for h in range(H):
            qv = q[b, h].astype(np.float64)                 # [D]
            m = meta[h // G, phys, 0, :].astype(np.float64)      # [P][D]
            M = meta[h // G, phys, 1, :].astype(np.float64)
            U = np.maximum(qv[None, :] * m, qv[None, :] * M)
            scores[b, h // G, :P] = np.maximum(scores[b, h // G, :P], U.sum(axis=1))
    return scores


# --------------------------------------------------------------------------
# Section 3.4: choose the K pages with the highest score
# --------------------------------------------------------------------------

def topk(scores, seq_lens, page_size, k_pages, keep_first=False, keep_newest=False):
    """Per (b, h): the K_b = min(k_pages, P_b) pages with the largest score.

    Ranking: score descending, then page index ascending (so of equal scores
    the lower page wins).  The chosen set is returned in ascending page order,
    padded with -1.  Returns (topk_idx int32 [B][H][k_pages], k_eff int32 [B]).

    keep_first / keep_newest (the paper selects purely by score; these are the
    two usual additions, kept optional): page 0 / the page of the newest token
    rank above every score, i.e. they take the first places of the K and the
    rest is filled by score."""
    B, H, _ = scores.shape
    idx = np.full((B, H, k_pages), -1, np.int32)
    k_eff = np.zeros(B, np.int32)
    for b in range(B):
        P = num_pages(seq_lens[b], page_size)
        K = min(int(k_pages), P)
        k_eff[b] = K
        for h in range(H):
            s = np.asarray(scores[b, h, :P])
            s = s + 0.0                                      # -0 and +0 rank equal
            kept = np.zeros(P, bool)                         # above every score, +inf included
            if keep_first:
                kept[0] = True
            if keep_newest:
                kept[P - 1] = True
            s[kept] = np.inf                                 # among themselves: by page index
            rank = np.lexsort((np.arange(P), -s, ~kept))     # last key is primary
            idx[b, h, :K] = np.sort(rank[:K])
    return idx, k_eff


# --------------------------------------------------------------------------
# Sections 3.1 and 3.4: ordinary attention restricted to the selected pages
# --------------------------------------------------------------------------

def sparse_decode(k_pool, v_pool, q, page_table, seq_lens, topk_idx, sm_scale):
    """o[b,h,:] = sum_j softmax_j(sm_scale * q.k_j) v_j over the valid tokens j
    of the selected pages; topk_idx=None selects every page (dense attention).

    Returns (out float64 [B][H][D], lse float64 [B][H]) with
    lse = log sum_j exp(sm_scale * q.k_j).

    With fewer KV heads than query heads (see estimate) query head h reads KV
    head h // G and the page list of that KV head."""
    B, H, D = q.shape
    S = k_pool.shape[2]
    G = H // k_pool.shape[1]
    assert G * k_pool.shape[1] == H
    out = np.zeros((B, H, D), np.float64)
    lse = np.zeros((B, H), np.float64)
    for b in range(B):
        L = int(seq_lens[b])
        P = num_pages(L, S)
        for h in range(H):
            if topk_idx is None:
                pages = np.arange(P)
            else:
                row = np.asarray(topk_idx[b, h // G])
                pages = row[row >= 0]
            phys = page_table[b, pages]
            keys = k_pool[phys, h // G].astype(np.float64).reshape(-1, D)     # [n*S][D]
            vals = v_pool[phys, h // G].astype(np.float64).reshape(-1, D)
            tok = (np.asarray(pages)[:, None] * S + np.arange(S)[None, :]).reshape(-1)
            ok = tok < L
            keys, vals = keys[ok], vals[ok]
            z = sm_scale * (keys @ q[b, h].astype(np.float64))
            zmax = z.max()
            w = np.exp(z - zmax)
            denom = w.sum()
            out[b, h] = (w[:, None] * vals).sum(axis=0) / denom
            lse[b, h] = zmax + np.log(denom)
    return out, lse


# --------------------------------------------------------------------------
# Section 3.5: memory-movement model
# --------------------------------------------------------------------------

def loaded_fraction(page_size: int, k_pages: int, total_pages: int) -> float:
    """Fraction of the KV cache Quest loads: 1/PageSize + K/PageNum."""
    return 1.0 / page_size + k_pages / total_pages
