"""Seeded synthetic inputs for the Quest decode hot path.

This module only draws random numbers and lays them out in the paged KV-cache
format; it contains none of the method's arithmetic (no min/max metadata, no
scores, no selection, no attention).  Both the CPU oracle's tests and the HIP
path's tests/bench take their inputs from here, so the two sides see the same
bytes without sharing any computation.

The workloads stand in for the long-context decode shapes the paper measures
(Llama-2-7B / LongChat-7B attention: 32 heads of dimension 128, fp16 KV cache,
page size 16, 32k context with a 2048-token budget; Section 4.3 of the paper).
The real prompts and model weights are not needed for the kernels' cost or
correctness: what matters is shape, dtype, a heavy-tailed per-channel key
distribution (a few outlier channels), slow drift of keys along the context
(so that pages differ and min/max boxes are informative), and a few planted
tokens strongly aligned with the query.

Layouts (numpy arrays, C order), mirrored by the device buffers:
  k_pool, v_pool : float16 [num_phys_pages][H][S][D]
  page_table     : int32   [B][max_pages]   logical page -> physical page id
  seq_lens       : int32   [B]
  q              : float16 [B][H][D]
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 20240610

# tensor ids that make every random stream distinct
_T_KEYS, _T_VALUES, _T_QUERY, _T_OUTLIER, _T_DRIFT, _T_PLANT, _T_PERM, _T_LENS, \
    _T_NEWK, _T_NEWV = range(10)


@dataclasses.dataclass(frozen=True)
class Workload:
    """One of the benchmark/parity configurations."""
    cid: int                      # configuration number (seeds the streams)
    name: str
    batch: int
    num_heads: int
    seq_lens: tuple               # tokens per sequence, len == batch
    token_budget: int
    planted_per_head: int
    head_dim: int = 128
    page_size: int = 16
    decode_steps: int = 0         # tokens appended in the timed/parity loop

    @property
    def k_pages(self) -> int:
        """Top-K page count K = floor(budget / page size), at least 1."""
        return max(1, self.token_budget // self.page_size)

    def pages_of(self, b: int) -> int:
        return -(-int(self.seq_lens[b]) // self.page_size)

    @property
    def max_pages(self) -> int:
        """Row stride of the page table: room for the decode steps as well."""
        longest = max(self.seq_lens) + self.decode_steps
        return -(-longest // self.page_size)


def _ragged_lengths(cid: int, batch: int, lo: int, hi: int) -> tuple:
    rng = np.random.default_rng([BASE_SEED, cid, _T_LENS])
    return tuple(int(x) for x in rng.integers(lo, hi + 1, size=batch))


def workload(cid: int, **overrides) -> Workload:
    """The five configurations of the benchmark definition (0 = tiny ... 4 = extreme)."""
    if cid == 0:
        w = Workload(0, "c0-tiny-1head-4k", 1, 1, (4096,), 512, 8, decode_steps=4)
    elif cid == 1:
        w = Workload(1, "c1-32head-32k-budget2048", 1, 32, (32768,), 2048, 64,
                     decode_steps=100)
    elif cid == 2:
        w = Workload(2, "c2-32head-128k", 1, 32, (131072,), 4096, 64, decode_steps=4)
    elif cid == 3:
        w = Workload(3, "c3-ragged-batch16", 16, 32,
                     _ragged_lengths(3, 16, 8192, 65536), 2048, 64, decode_steps=64)
    elif cid == 4:
        w = Workload(4, "c4-32head-512k", 1, 32, (524288,), 4096, 256, decode_steps=2)
    else:
        raise ValueError(f"unknown configuration {cid}")
    return dataclasses.replace(w, **overrides) if overrides else w


def _rng(cid, b, h, tensor_id, extra=0):
    return np.random.default_rng([BASE_SEED, cid, b, h, tensor_id, extra])


def gen_query(w: Workload, step: int = 0) -> np.ndarray:
    """q ~ N(0, I), fp16 [B][H][D]; a fresh draw per decode step."""
    q = np.empty((w.batch, w.num_heads, w.head_dim), np.float16)
    for b in range(w.batch):
        for h in range(w.num_heads):
            q[b, h] = _rng(w.cid, b, h, _T_QUERY, step).standard_normal(
                w.head_dim, dtype=np.float32).astype(np.float16)
    return q


def gen_new_token(w: Workload, step: int):
    """Key/value of the token appended at decode step `step`: fp16 [B][H][D] each.

    Keys continue the drift of the last prompt page so the new page looks like
    its neighbours; values are N(0, I)."""
    k = np.empty((w.batch, w.num_heads, w.head_dim), np.float16)
    v = np.empty_like(k)
    for b in range(w.batch):
        for h in range(w.num_heads):
            scale = _channel_scale(w, b, h)
            drift = _drift(w, b, h, w.pages_of(b))[-1]
            kk = _rng(w.cid, b, h, _T_NEWK, step).standard_normal(w.head_dim, dtype=np.float32)
            k[b, h] = ((kk + drift) * scale).astype(np.float16)
            v[b, h] = _rng(w.cid, b, h, _T_NEWV, step).standard_normal(
                w.head_dim, dtype=np.float32).astype(np.float16)
    return k, v


def _channel_scale(w: Workload, b: int, h: int) -> np.ndarray:
    """4 distinct outlier channels per head scaled x8, the rest x1."""
    s = np.ones(w.head_dim, np.float32)
    ch = _rng(w.cid, b, h, _T_OUTLIER).choice(w.head_dim, size=min(4, w.head_dim), replace=False)
    s[ch] = 8.0
    return s


def _drift(w: Workload, b: int, h: int, pages: int) -> np.ndarray:
    """Per-page random walk d_0 = 0, d_p = d_{p-1} + N(0, 0.3^2 I): float32 [pages][D]."""
    steps = _rng(w.cid, b, h, _T_DRIFT).standard_normal((pages, w.head_dim), dtype=np.float32)
    steps *= np.float32(0.3)
    steps[0] = 0.0
    return np.cumsum(steps, axis=0, dtype=np.float32)


def planted_positions(w: Workload, b: int, h: int) -> np.ndarray:
    L = int(w.seq_lens[b])
    n = min(w.planted_per_head, L)
    return np.sort(_rng(w.cid, b, h, _T_PLANT).choice(L, size=n, replace=False))


def gen_head_kv(w: Workload, b: int, h: int, q0: np.ndarray):
    """Keys and values of one (sequence, head): fp16 [L][D] each.

    keys   : (N(0, I) + d_page) * outlier_scale; planted tokens get 3 q0/|q0|
    values : N(0, I)
    """
    L, S, D = int(w.seq_lens[b]), w.page_size, w.head_dim
    P = w.pages_of(b)
    k = _rng(w.cid, b, h, _T_KEYS).standard_normal((L, D), dtype=np.float32)
    drift = _drift(w, b, h, P)
    k += np.repeat(drift, S, axis=0)[:L]
    k *= _channel_scale(w, b, h)[None, :]
    qf = q0.astype(np.float32)
    k[planted_positions(w, b, h)] = 3.0 * qf / np.linalg.norm(qf)
    v = _rng(w.cid, b, h, _T_VALUES).standard_normal((L, D), dtype=np.float32)
    return k.astype(np.float16), v.astype(np.float16)


def make_page_table(w: Workload, permute: bool, spare_pages: int = 2):
    """Logical -> physical page map.

    Returns (page_table int32 [B][max_pages], num_phys_pages).  Every logical
    page up to max_pages of every sequence gets its own physical page (so the
    decode steps have somewhere to append); `spare_pages` unmapped physical
    pages are left over as canaries.  permute=False gives the identity map used
    for timing; permute=True shuffles physical ids (seeded) to exercise the
    gather."""
    B, mp = w.batch, w.max_pages
    per_seq = [-(-(int(L) + w.decode_steps) // w.page_size) for L in w.seq_lens]
    total = int(sum(per_seq)) + spare_pages
    ids = np.arange(total, dtype=np.int32)
    if permute:
        ids = np.random.default_rng([BASE_SEED, w.cid, _T_PERM]).permutation(total).astype(np.int32)
    table = np.full((B, mp), -1, np.int32)
    at = 0
    for b in range(B):
        table[b, :per_seq[b]] = ids[at:at + per_seq[b]]
        at += per_seq[b]
    return table, total


def fill_pools(w: Workload, page_table: np.ndarray, num_phys_pages: int,
               stale_fill: float = float("nan"), threads: int = 8, progress=None):
    """Generate K/V for every (sequence, head) and scatter into paged pools.

    Slots that hold no valid token (tail of a partial last page, pages reserved
    for later decode steps, spare pages) are filled with `stale_fill` (NaN by
    default) so that any read of a stale slot poisons the result.
    progress(done, total), if given, is called as (sequence, head) pairs are finished.
    Returns (k_pool, v_pool, q0) with q0 = the step-0 query fp16 [B][H][D]."""
    H, S, D = w.num_heads, w.page_size, w.head_dim
    k_pool = np.full((num_phys_pages, H, S, D), stale_fill, np.float16)
    v_pool = np.full((num_phys_pages, H, S, D), stale_fill, np.float16)
    q0 = gen_query(w, 0)

    def one(bh):
        b, h = bh
        L = int(w.seq_lens[b])
        P = w.pages_of(b)
        k, v = gen_head_kv(w, b, h, q0[b, h])
        full = L // S
        phys = page_table[b, :P]
        if full:
            k_pool[phys[:full], h] = k[:full * S].reshape(full, S, D)
            v_pool[phys[:full], h] = v[:full * S].reshape(full, S, D)
        if full < P:
            n = L - full * S
            k_pool[phys[full], h, :n] = k[full * S:]
            v_pool[phys[full], h, :n] = v[full * S:]

    jobs = [(b, h) for b in range(w.batch) for h in range(H)]
    if threads > 1 and len(jobs) > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            for n, _ in enumerate(ex.map(one, jobs)):
                if progress is not None:
                    progress(n + 1, len(jobs))
    else:
        for n, j in enumerate(jobs):
            one(j)
            if progress is not None:
                progress(n + 1, len(jobs))
    return k_pool, v_pool, q0
