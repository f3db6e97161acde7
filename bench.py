#!/usr/bin/env python3
"""Benchmark of the Quest decode hot path on one MI355X.

A step is one layer-step of decode on the LongChat-7B-shaped workload
(config 1: batch 1, 32 heads x 128, fp16 KV, 32k context, page 16, token
budget 2048): append one token (KV write + min/max update), estimate page
criticality, select the top 128 pages, sparse paged attention over them.
Steps rotate over `--layers` distinct layer buffers, as the layers of a model
do, so metadata and KV pages come from HBM rather than from the 256 MB
last-level cache.  The K timed steps are captured once into a HIP graph and
replayed, so host launch overhead is not what is measured.

Prints ONE JSON line: value = microseconds per layer-step; next to it the
achieved HBM GB/s on the bytes the method has to touch (metadata + selected KV
pages, Section 3.5 of the paper), the library's own dense path (all pages) on
the same buffers, the roofline entry of the dominant kernel and the CPU oracle
timed on the host cores.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=16, help="distinct layer buffers to rotate over")
    ap.add_argument("--config", type=int, default=1, help="workload id (1 = headline)")
    ap.add_argument("--page-size", type=int, default=0,
                    help="tokens per page (8, 16, 32, 64) instead of the workload's own; same "
                         "context and token budget (the page-size sweep of the paper's Figure 8)")
    ap.add_argument("--repeats", type=int, default=5, help="graph replays; the median is reported")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="grouped-query attention: KV heads (a divisor of the workload's heads); "
                         "the workload's heads stay the query heads.  Implies --no-cpu-baseline")
    ap.add_argument("--token-budget", type=int, default=0,
                    help="token budget instead of the workload's own (K = budget / page size)")
    ap.add_argument("--batch", type=int, default=0,
                    help="that many copies of the workload's (single) sequence in one batch: the "
                         "throughput regime.  Implies --no-cpu-baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-yardsticks", action="store_true",
                    help="skip the plain-read and bare-gather kernels timed next to the library's")
    ap.add_argument("--eager", action="store_true", help="also time eager (per-call) launches")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); the path shards over "
              "heads and sequences without communication, each GPU runs this same step on its share",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2406_10774_amd import binding as Q, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n_total = args.warmup + args.steps
    n_layers = args.layers
    visits = -(-n_total // n_layers)                      # appends per layer buffer
    over = {"page_size": args.page_size} if args.page_size else {}
    if args.token_budget:
        over["token_budget"] = args.token_budget
    if args.batch:
        base = synth.workload(args.config)
        assert base.batch == 1, "--batch replicates a single-sequence workload"
        over["batch"] = args.batch
        over["seq_lens"] = tuple(base.seq_lens) * args.batch
        args.no_cpu_baseline = True
    wq = synth.workload(args.config, decode_steps=visits + 1, **over)   # query side
    Hq = wq.num_heads
    if args.kv_heads:
        assert Hq % args.kv_heads == 0, "--kv-heads must divide the number of heads"
        over["num_heads"] = args.kv_heads
        args.no_cpu_baseline = True
    w = synth.workload(args.config, decode_steps=visits + 1, **over)    # KV side
    B, H, S, D, K = w.batch, w.num_heads, w.page_size, w.head_dim, w.k_pages
    scale = 1.0 / math.sqrt(D)

    # ---------------------------------------------------------------- inputs
    t0 = time.time()
    table, N = synth.make_page_table(w, permute=False)
    last = [time.time()]

    def progress(done, total):                            # long set-ups say that they are alive
        if time.time() - last[0] > 20 or done == total:
            last[0] = time.time()
            print(f"bench.py: generated {done} of {total} (sequence, head) pairs", file=sys.stderr, flush=True)

    k_pool, v_pool, _ = synth.fill_pools(w, table, N, stale_fill=0.0, threads=16, progress=progress)
    lens0 = np.array(w.seq_lens, np.int32)

    def dev16(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(dev).view(torch.float16)

    k0, v0 = dev16(k_pool), dev16(v_pool)
    pt = torch.from_numpy(table).to(dev)
    # step i visits layer i % n_layers for the (i // n_layers + 1)-th time
    lens_steps = np.stack([lens0 + (i // n_layers + 1) for i in range(n_total)]).astype(np.int32)
    lens_dev = torch.from_numpy(lens_steps).to(dev)
    lens0_dev = torch.from_numpy(lens0).to(dev)
    q_all = dev16(np.stack([synth.gen_query(wq, i) for i in range(n_total)]))
    new_kv = []
    for i in range(n_total):
        new_kv.append(synth.gen_new_token(w, i))
        if time.time() - last[0] > 20:
            last[0] = time.time()
            print(f"bench.py: new tokens of step {i + 1} of {n_total} generated", file=sys.stderr, flush=True)
    kn_all = dev16(np.stack([k for k, _ in new_kv]))
    vn_all = dev16(np.stack([v for _, v in new_kv]))

    layers = []
    for l in range(n_layers):
        kp = k0 if l == 0 else k0.clone()
        vp = v0 if l == 0 else v0.clone()
        meta = torch.zeros((H, N, 2, D), dtype=torch.float16, device=dev)
        Q.quest_build_meta(Q.Cache(kp, vp, meta, pt, lens0_dev))
        layers.append((kp, vp, meta))
        if time.time() - last[0] > 20:
            last[0] = time.time()
            print(f"bench.py: layer buffer {l + 1} of {n_layers} on the device", file=sys.stderr, flush=True)
    caches = [Q.Cache(*layers[i % n_layers], pt, lens_dev[i], num_heads=Hq) for i in range(n_total)]
    scores = torch.zeros((B, H, table.shape[1]), dtype=torch.float32, device=dev)
    idx = torch.zeros((B, H, K), dtype=torch.int32, device=dev)
    out = torch.zeros((B, Hq, D), dtype=torch.float32, device=dev)
    ws_bytes = max(Q.quest_workspace_bytes(caches[0], K), Q.quest_workspace_bytes(caches[0], 0), 4)
    ws = torch.zeros(ws_bytes // 4, dtype=torch.float32, device=dev)
    ws_step = torch.zeros(max(Q.quest_step_workspace_bytes(caches[0], K), 8) // 4, dtype=torch.int32,
                          device=dev)
    torch.cuda.synchronize()
    gen_s = time.time() - t0

    # ------------------------------------------------------------- the step
    def sparse_step(i):                                   # three launches
        c = caches[i]
        Q.quest_append_estimate(c, kn_all[i], vn_all[i], True, q_all[i], scores)
        Q.quest_topk(c, scores, K, idx, None)
        Q.quest_sparse_decode(c, q_all[i], idx, K, scale, out, None, ws)

    def sparse_step_separate(i):                          # one launch per call of the method
        c = caches[i]
        Q.quest_append_meta(c, kn_all[i], vn_all[i], True)
        Q.quest_estimate(c, q_all[i], scores)
        Q.quest_topk(c, scores, K, idx, None)
        Q.quest_sparse_decode(c, q_all[i], idx, K, scale, out, None, ws)

    def two_launch_step(i):                               # estimate launch, then selection + attention launch
        Q.quest_decode_step(caches[i], kn_all[i], vn_all[i], True, q_all[i], K, scale,
                            scores, idx, out, ws_step)

    def dense_step(i):
        c = caches[i]
        Q.quest_append_meta(c, kn_all[i], vn_all[i], True)
        Q.quest_sparse_decode(c, q_all[i], None, 0, scale, out, None, ws)

    def capture(fn, indices):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in indices:
                fn(i)
        return g

    def time_graph(g, repeats):
        """Median wall-clock seconds of one replay, synchronised on both sides."""
        times = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t = time.perf_counter()
            g.replay()
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t)
        return float(np.median(times)), times

    def time_graph_events(g, repeats):
        """Median GPU seconds (HIP events on the launch stream) of one replay."""
        times = []
        for _ in range(repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e-3)
        return float(np.median(times))

    timed = list(range(args.warmup, n_total))
    for i in range(args.warmup):                          # untimed warm-up, eager
        sparse_step(i)
    torch.cuda.synchronize()
    g_sparse = capture(sparse_step, timed)
    g_sparse.replay()
    sec, all_sec = time_graph(g_sparse, args.repeats)
    us_step = sec / args.steps * 1e6
    us_step_events = time_graph_events(g_sparse, args.repeats) / args.steps * 1e6

    g_sep = capture(sparse_step_separate, timed)
    g_sep.replay()
    sep_us = time_graph(g_sep, max(3, args.repeats // 2))[0] / args.steps * 1e6

    g_two = capture(two_launch_step, timed)
    g_two.replay()
    two_us = time_graph(g_two, args.repeats)[0] / args.steps * 1e6
    two_us_events = time_graph_events(g_two, args.repeats) / args.steps * 1e6
    # headline: the faster of the ways the library offers to run the complete step
    three_us = us_step
    calls = "quest_append_estimate, quest_topk, quest_sparse_decode (three launches)"
    # the library's own rule (quest.h): the attention launch selects its pages itself for
    # rows of at most 4096 pages and lists of at most 2048; else the call is three launches
    selects_inside = table.shape[1] <= 4096 and K <= 2048
    one_call = two_us < us_step
    two_launches = one_call and selects_inside
    if one_call:
        us_step, us_step_events = two_us, two_us_events
        calls = ("quest_decode_step (two launches: estimate; selection + attention)" if selects_inside
                 else "quest_decode_step (one call; estimate, selection and attention as launches of their own)")

    g_dense = capture(dense_step, timed)
    g_dense.replay()
    dense_sec, _ = time_graph(g_dense, max(3, args.repeats // 2))
    dense_us = dense_sec / args.steps * 1e6

    eager_us = None
    if args.eager:
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in timed:
            sparse_step(i)
        torch.cuda.synchronize()
        eager_us = (time.perf_counter() - t) / args.steps * 1e6

    # bytes the method has to move per step: metadata of every page + selected KV pages
    pages_steps = [int(sum(-(-int(x) // S) for x in lens_steps[i])) for i in timed]
    meta_bytes = float(np.mean([H * p * 512 for p in pages_steps]))
    ksel = [sum(min(K, -(-int(x) // S)) for x in lens_steps[i]) for i in timed]
    page_bytes = 2 * S * D * 2                            # keys + values of one (page, head)
    kv_bytes = float(np.mean([H * k * page_bytes for k in ksel]))
    dense_bytes = float(np.mean([H * p * page_bytes for p in pages_steps]))
    step_bytes = meta_bytes + kv_bytes
    gbps = step_bytes / (us_step * 1e-6) / 1e9

    # ------------------------------------------------ per-kernel launch times
    def kernel_us(fn, reps=4):
        g = capture(fn, timed * reps)
        g.replay()
        return time_graph_events(g, 3) / (len(timed) * reps) * 1e6

    k_est = kernel_us(lambda i: Q.quest_estimate(caches[i], q_all[i], scores))
    k_appest = kernel_us(lambda i: Q.quest_append_estimate(caches[i], kn_all[i], vn_all[i], True,
                                                           q_all[i], scores))
    k_topk = kernel_us(lambda i: Q.quest_topk(caches[i], scores, K, idx, None))
    # rows long enough for the selection in two stages (two launches: per-chunk candidates, then
    # the K best of those), which quest_topk runs when the caller brings the workspace for it
    topk_ws_bytes = Q.quest_topk_workspace_bytes(caches[0], K)
    k_topk2 = None
    if topk_ws_bytes:
        topk_ws = torch.zeros(topk_ws_bytes, dtype=torch.uint8, device=dev)
        k_topk2 = kernel_us(lambda i: Q.quest_topk(caches[i], scores, K, idx, None, topk_ws))
    k_dec = kernel_us(lambda i: Q.quest_sparse_decode(caches[i], q_all[i], idx, K, scale, out, None, ws))
    k_app = kernel_us(lambda i: Q.quest_append_meta(caches[i], kn_all[i], vn_all[i], True))
    k_dense = kernel_us(lambda i: Q.quest_sparse_decode(caches[i], q_all[i], None, 0, scale, out,
                                                        None, ws), reps=1)
    # the attention launch that selects its own pages (the second launch of the one-call step)
    k_seldec = kernel_us(lambda i: Q.quest_select_decode(caches[i], q_all[i], scores, K, scale, idx,
                                                         out, workspace=ws_step)) \
        if selects_inside else float("nan")
    score_bytes = float(np.mean([H * p * 4 for p in pages_steps]))
    kernels = {
        "append_meta_us": round(k_app, 3),
        "estimate_us": round(k_est, 3), "estimate_gbps": round(meta_bytes / k_est / 1e3, 1),
        "append_estimate_us": round(k_appest, 3),
        "append_estimate_gbps": round(meta_bytes / k_appest / 1e3, 1),
        "topk_us": round(k_topk, 3),
        "topk_two_stage_us": None if k_topk2 is None else round(k_topk2, 3),
        "sparse_decode_us": round(k_dec, 3), "sparse_decode_gbps": round(kv_bytes / k_dec / 1e3, 1),
        "select_decode_us": round(k_seldec, 3) if selects_inside else None,
        "select_decode_gbps": round((kv_bytes + score_bytes) / k_seldec / 1e3, 1) if selects_inside else None,
        "dense_decode_us": round(k_dense, 3), "dense_decode_gbps": round(dense_bytes / k_dense / 1e3, 1),
    }
    if k_appest >= k_dec:
        dom, dom_us, dom_bytes = "quest_append_estimate", k_appest, meta_bytes
    else:
        dom, dom_us, dom_bytes = "quest_sparse_decode", k_dec, kv_bytes
    if two_launches and k_seldec > k_appest:                # selection + attention in one kernel
        dom, dom_us, dom_bytes = "quest_select_decode", k_seldec, kv_bytes + score_bytes
    achieved = dom_bytes / dom_us / 1e3
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                # the counters were collected on the headline configuration only; this run does
                # not measure them (the profiler cannot run inside it): the figure is the one
                # recorded under profiles/ for the same kernel and launch shape
                "traffic": load_traffic(dom) if args.config == 1 and not (
                    args.batch or args.page_size or args.kv_heads or args.token_budget) else None,
                "traffic_source": "profiles/hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                                  "per dispatch, scaled by a copy kernel of known size)"}

    roofline["frac_of_yardstick"] = None
    yard = None
    if not args.no_yardsticks:
        yard = yardsticks(torch, layers, idx, pt, H, S, D, args.steps)
        # the dominant kernel against the machine's own rate on its access pattern with no
        # arithmetic: a plain scan for the estimate, a bare gather for the attention
        ref = yard["stream_gbps_32mib"] if dom == "quest_append_estimate" else yard["gather_gbps"]
        if ref:
            roofline["frac_of_yardstick"] = round(achieved / ref, 4)
    build = time_build_meta(torch, Q, layers, pt, lens0_dev, lens0, H, S, D)
    kernels.update(build)

    # ---------------------------------------------------------- CPU baseline
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(w, table, k_pool, v_pool, lens0, scale)

    line = {
        "metric": "sparse decode attn \u00b5s/layer-step + achieved HBM GB/s (32 heads, 32k ctx, budget 2048)",
        "value": round(us_step, 3), "unit": "us/layer-step",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_step * 1e-3, 6), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "storage_dtype": "f16", "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "heads": Hq, "kv_heads": H, "head_dim": D,
                   "page_size": S,
                   "context": int(lens0.max()), "token_budget": w.token_budget, "k_pages": K,
                   "layer_buffers": n_layers, "launch": "hip-graph replay of the timed steps",
                   "calls_per_step": calls},
        "hbm_gbps": round(gbps, 1), "hbm_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
        "bytes_per_step": int(step_bytes), "us_per_step_gpu_events": round(us_step_events, 3),
        "separate_calls_us_per_step": round(sep_us, 3),
        "three_launch_us_per_step": round(three_us, 3),
        "decode_step_call_us_per_step": round(two_us, 3),
        "dense_us_per_step": round(dense_us, 3),
        "dense_hbm_gbps": round(dense_bytes / (dense_us * 1e-6) / 1e9, 1),
        "speedup_vs_own_dense": round(dense_us / us_step, 3),
        "eager_us_per_step": None if eager_us is None else round(eager_us, 3),
        "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu,
        "yardsticks": yard, "host_nproc": os.cpu_count(),
        "setup_s": round(gen_s, 1),
    }
    print(json.dumps(line))


def _graph_us(torch, fn, n, repeats=3):
    """Median GPU microseconds per call of fn(i), i < n, captured once and replayed."""
    fn(0)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(n):
            fn(i)
    g.replay()
    times = []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / n)
    return float(np.median(times))


def yardsticks(torch, layers, idx, pt, H, S, D, n):
    """What the machine does on the step's access patterns with no arithmetic, measured in
    this run on the same buffers (rotating over the layers like the step does): a launch
    floor, plain scans of the metadata table and of K + V, and a gather of the selected
    (page, head) blocks through a list in the attention's launch shape."""
    path = os.path.join(ROOT, "paper_2406_10774_amd", "libquest_yardstick.so")
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2406_10774_amd.build`")
    lib = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    lib.yardstick_empty.argtypes = [vp]
    lib.yardstick_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, ctypes.c_int, vp, vp]
    lib.yardstick_gather.argtypes = [vp, vp, vp, ctypes.c_int, ctypes.c_int, vp, vp]
    sink = torch.zeros(4, dtype=torch.int32, device=idx.device)
    nl = len(layers)

    def stream():
        return vp(torch.cuda.current_stream().cuda_stream)

    def ok(r):
        assert r == 0, "yardstick launch failed"

    out = {}
    out["empty_launch_us"] = round(_graph_us(torch, lambda i: ok(lib.yardstick_empty(stream())), n), 3)
    meta_bytes = layers[0][2].numel() * 2
    kv_bytes = layers[0][0].numel() * 2
    for nt in (0, 1):
        tag = "_nt" if nt else ""
        us = _graph_us(torch, lambda i: ok(lib.yardstick_read(
            vp(layers[i % nl][2].data_ptr()), meta_bytes, None, 0, nt, vp(sink.data_ptr()), stream())), n)
        out["stream_us_meta" + tag] = round(us, 3)
        out["stream_gbps_meta" + tag] = round(meta_bytes / us / 1e3, 1)
        us = _graph_us(torch, lambda i: ok(lib.yardstick_read(
            vp(layers[i % nl][0].data_ptr()), kv_bytes, vp(layers[i % nl][1].data_ptr()), kv_bytes, nt,
            vp(sink.data_ptr()), stream())), max(4, n // 8))
        out["stream_us_kv" + tag] = round(us, 3)
        out["stream_gbps_kv" + tag] = round(2 * kv_bytes / us / 1e3, 1)
    out["meta_table_mib"] = round(meta_bytes / 2 ** 20, 1)
    out["kv_pools_mib"] = round(2 * kv_bytes / 2 ** 20, 1)
    # the better of the two load kinds is the yardstick (the library's kernels use the
    # non-temporal kind); named for the sizes they have at the headline configuration
    out["stream_gbps_32mib"] = max(out["stream_gbps_meta"], out["stream_gbps_meta_nt"])
    out["stream_gbps_512mib"] = max(out["stream_gbps_kv"], out["stream_gbps_kv_nt"])
    out["gather_gbps"] = None
    if S * D * 2 == 4096:
        # the page list of the last step, as block ids into the pools: (physical page, head)
        B, Hk, K = idx.shape
        lp = idx.clamp(min=0).long()                                    # [B][H][K]
        phys = torch.gather(pt.long().unsqueeze(1).expand(B, Hk, pt.shape[1]), 2, lp)
        blocks = (phys * Hk + torch.arange(Hk, device=idx.device).view(1, Hk, 1))[idx >= 0]
        blocks = blocks.to(torch.int32).contiguous()
        n_blk = int(blocks.numel())
        for nt in (0, 1):
            us = _graph_us(torch, lambda i: ok(lib.yardstick_gather(
                vp(layers[i % nl][0].data_ptr()), vp(layers[i % nl][1].data_ptr()),
                vp(blocks.data_ptr()), n_blk, nt, vp(sink.data_ptr()), stream())), n)
            out["gather_us" + ("_nt" if nt else "")] = round(us, 3)
            out["gather_gbps" + ("_nt" if nt else "_plain")] = round(n_blk * 8192 / us / 1e3, 1)
        out["gather_blocks"] = n_blk
        out["gather_gbps"] = max(out["gather_gbps_plain"], out["gather_gbps_nt"])
    return out


def time_build_meta(torch, Q, layers, pt, lens_dev, lens, H, S, D):
    """quest_build_meta over all pages of every layer buffer (the prefill side of the path):
    microseconds per call and GB/s on the keys it has to read."""
    caches = [Q.Cache(kp, vp_, meta, pt, lens_dev) for kp, vp_, meta in layers]
    us = _graph_us(torch, lambda i: Q.quest_build_meta(caches[i % len(caches)]), max(len(caches), 8))
    pages = int(sum(-(-int(x) // S) for x in lens))
    read = H * pages * S * D * 2
    written = H * pages * 2 * D * 2
    return {"build_meta_us": round(us, 3), "build_meta_gbps": round(read / us / 1e3, 1),
            "build_meta_read_written_gbps": round((read + written) / us / 1e3, 1),
            "build_meta_read_mib": round(read / 2 ** 20, 1)}


def load_traffic(kernel):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a copy kernel of known size); kept as a small text file
    next to the profile summaries.  None if it has not been measured."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for ln in open(path):
        parts = ln.split()
        if len(parts) >= 2 and parts[0] == kernel:
            return float(parts[1])
    return None


def cpu_baseline(w, table, k_pool, v_pool, lens0, scale):
    """The oracle, as it stands, on the host: full layer-steps of the same workload."""
    from oracle import quest_oracle as O
    from paper_2406_10774_amd import synth
    try:
        from threadpoolctl import threadpool_limits
    except ImportError:                                   # pragma: no cover
        threadpool_limits = None
    S = w.page_size
    meta = O.build_meta(k_pool, table, lens0)
    n = 3
    cur = lens0.copy()

    def run():
        nonlocal meta, cur
        t = time.perf_counter()
        for i in range(n):
            q = synth.gen_query(w, 1000 + i)
            k_new, v_new = synth.gen_new_token(w, 1000 + i)
            t_in = time.perf_counter()
            cur = cur + 1
            O.append_kv(k_pool, v_pool, k_new, v_new, table, cur)
            meta = O.append_meta(meta, k_new, table, cur, S)
            sc = O.estimate(meta, q, table, cur, S)
            idx, _ = O.topk(sc, cur, S, w.k_pages)
            O.sparse_decode(k_pool, v_pool, q, table, cur, idx, scale)
            run.acc += time.perf_counter() - t_in
        return time.perf_counter() - t
    run.acc = 0.0
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            run()
    else:
        run()
    return {"value": round(run.acc / n * 1e6, 1), "unit": "us/layer-step", "cores": 1,
            "kind": "oracle", "sample": f"{n} full layer-steps of {w.name} (numpy float64, 1 thread)"}


if __name__ == "__main__":
    main()
