#!/usr/bin/env python3
"""Benchmark of the top-k attention decode hot path on one MI355X.

A step is one topk_attn_decode call (key scan -> exact top-k -> softmax-weighted gather)
over one layer of the N = 1M configuration (32 query heads, 8 KV heads, d = 128, fp16,
k = 16384).  The cache is resident in HBM before timing starts; steps rotate over
several layers so every scan reads HBM-cold keys.  Prints one JSON line.

--workload c1 | c2 | c4 | c5 times the other configurations the same way (they are parity-test
cases, not the metric's workload): c1 the small fp32 case (launch-bound), c2 one 128k-token layer, c4 sixteen sequences of 256k
tokens per step, c5 one layer of the 32-layer 512k-token cache (all 32 resident, a step is
one layer's decode).  --workload c6 --pages times the sub-linear search through the page index
on the cache with topical runs (the scan reads only the pages whose bound reaches the threshold).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published


def measured_traffic(kernel: str, workload: str):
    """HBM bytes one launch of `kernel` moves at `workload`, as the committed rocprofv3 counter summary
    states it (FETCH_SIZE + WRITE_SIZE, calibrated against copy kernels of known size); None when the
    summary does not cover that kernel and workload."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "decode_c3_hbm_counters.md")
    try:
        with open(path) as f:
            for line in f:
                m = re.match(r"traffic: kernel=(\S+) workload=(\S+) bytes_per_launch=(\S+)", line.strip())
                if m and m.group(1) == kernel and m.group(2) == workload:
                    return float(m.group(3))
    except OSError:
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--layers", type=int, default=4, help="distinct resident layers the steps rotate over")
    ap.add_argument("--tokens", type=int, default=0, help="override N (debug only; invalidates the metric)")
    ap.add_argument("--queries", type=int, default=1,
                    help="queries per step (a causal chunk through topk_attn_decode_multi); 1 is the metric's workload")
    ap.add_argument("--index", action="store_true",
                    help="approximate search through the int8 key index (exact refinement); not the metric's workload")
    ap.add_argument("--window", type=int, default=0,
                    help="recent tokens always attended and left out of the search (topk_attn_decode_window); not the metric's workload")
    ap.add_argument("--pages", action="store_true",
                    help="sub-linear search through the page index (exact with --beta 1); not the metric's workload")
    ap.add_argument("--beta", type=float, default=1.0, help="scale of the page radius in the page bound (--pages)")
    ap.add_argument("--sigma", type=float, default=0.0, help="spread of the keys of a run around its centroid (c6; 0 = the recipe's)")
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5", "c6"],
                    help="c3 is the metric's workload; the others are timed the same way for reference")
    ap.add_argument("--k", type=int, default=0, help="override k (c4 is swept over 256, 1024, 4096 in the tests)")
    ap.add_argument("--force-redo", action="store_true",
                    help="worst case of the filtered path: every head is redone exactly (not the metric's workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2502_06766_amd import topk_attn as ta
    from paper_2502_06766_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda", 0)
    w = {"c1": wl.C1, "c2": wl.C2, "c3": wl.C3, "c4": wl.C4, "c5": wl.C5, "c6": wl.C6}[args.workload]
    default = args.workload == "c3" and not args.tokens and not args.k and not args.force_redo and not args.pages and not args.window   # the metric's workload as it stands
    if args.tokens:
        w = w.scaled(args.tokens)
    N, k, d, Hq, Hkv, B = w.n_tokens, args.k or w.k, w.head_dim, w.n_q_heads, w.n_kv_heads, w.n_seqs
    # layers resident at once: enough distinct key bytes that no scan finds its keys in a cache
    L = max(1, {"c1": 8, "c2": 8, "c3": args.layers, "c4": 1, "c5": 32, "c6": args.layers}[args.workload])

    t0 = time.time()
    if args.workload == "c6":
        sigma = args.sigma or wl.CLUSTER_SIGMA
        q, K, V = (wl.quantize(a, w.dtype) for a in wl.make_clustered(w, args.seed, sigma, threads=16))
    else:
        q, K, V = wl.make_quantized(w, args.seed, threads=16)
    gen_s = time.time() - t0

    M = max(1, args.queries)
    cache = ta.TopkAttnCache(L, B, Hq, Hkv, d, N, k, w.dtype, max_queries=M, max_window=args.window,
                             index_kind=ta.INDEX_INT8 if args.index else ta.INDEX_PAGES if args.pages else ta.INDEX_NONE)
    if args.index:
        cache.set_path(ta.PATH_INDEX)
    if args.pages:
        cache.set_path(ta.PATH_PAGES)
        ta.topk_attn_set_page_bound_scale(cache.h, args.beta)
    if args.force_redo:
        ta.topk_attn_debug_force_redo(cache.h, True)

    def to_dev(a):
        return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16) if w.dtype == wl.BF16 else \
            torch.from_numpy(a).to(dev)

    Kd, Vd = to_dev(K), to_dev(V)
    for layer in range(L):
        for b in range(B):   # same distribution, different addresses and row order
            sh = 7919 * (layer * B + b)
            cache.append(layer, b, torch.roll(Kd, sh, 1) if sh else Kd, torch.roll(Vd, sh, 1) if sh else Vd,
                         head_major=True)
    del Kd, Vd
    if M > 1:
        q = wl.make_query_chunk(q, w.dtype, M, args.seed)
    qd = to_dev(q)[None].expand(B, *q.shape).contiguous()
    out = torch.empty((B, M, Hq, d), dtype=torch.float32, device=dev)
    idx = torch.empty((B, M, Hq, k), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    torch.cuda.synchronize()

    def step(i):
        if M == 1 and args.window:
            ta.topk_attn_decode_window(cache.h, i % L, qd.data_ptr(), k, args.window, out.data_ptr(), idx.data_ptr(), 0, 0, stream)
        elif M == 1:
            ta.topk_attn_decode(cache.h, i % L, qd.data_ptr(), k, out.data_ptr(), idx.data_ptr(), 0, 0, stream)
        else:
            ta.topk_attn_decode_multi(cache.h, i % L, qd.data_ptr(), M, True, k, args.window, out.data_ptr(), idx.data_ptr(),
                                      0, 0, stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    fallbacks = cache.last_fallbacks()
    pages_read, pages_total = ta.topk_attn_last_pages_read(cache.h)

    ta.topk_attn_set_scan_timing(cache.h, True)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(args.steps):
        step(i)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps
    scan_ms_total, n_scan = ta.topk_attn_scan_time(cache.h)
    ta.topk_attn_set_scan_timing(cache.h, False)
    scan_ms = scan_ms_total / max(1, n_scan)

    # spread of the single steps, from a second pass with an event between steps (the events
    # cost a little, so this pass is not the one the metric is taken from)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))

    # streaming-read ceiling over the same key bytes (128-bit loads, nothing else)
    sink = torch.zeros(16384, dtype=torch.int32, device=dev)
    e = 4 if w.dtype == wl.F32 else 2
    k_bytes = B * Hkv * N * d * e          # the key bytes of one layer
    probe_ms = []
    for i in range(L * 3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ta.topk_attn_read_probe(cache.kv.data_ptr() + (i % L) * k_bytes, k_bytes, sink.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        probe_ms.append(e0.elapsed_time(e1))
    probe_gbps = k_bytes / (min(probe_ms[min(L, len(probe_ms) - 1):]) * 1e-3) / 1e9

    alg_bytes = k_bytes + B * M * (Hq * k * d * e + Hq * d * (e + 4) + Hq * k * 4)
    keys_per_s = B * Hkv * N / (ms_per_step * 1e-3)
    # every key is needed once per launch, however many blocks of (query, head) rows walk over it
    scan_bytes = k_bytes
    if args.index and M == 1:
        scan_bytes = B * Hkv * N * (d + 4)                      # int8 codes and one fp32 scale per key
    if args.pages and M == 1:                                   # the pages kept, and one mask bit per page
        scan_bytes = pages_read * 64 * d * e + pages_total // 8
    scan_gbps = scan_bytes / (scan_ms * 1e-3) / 1e9
    scan_kernel = "scan_generic_kernel<full>" if w.dtype == wl.F32 else "scan_rows_kernel<filter>" if M > 1 else \
        "scan8_kernel<filter>" if args.index else "scan_mfma_kernel<filter,paged>" if args.pages else "scan_mfma_kernel<filter>"

    cpu = None
    if not args.no_cpu_baseline and M == 1 and not args.index:
        from oracle import c_oracle
        t0 = time.perf_counter()
        c_oracle.topk_attention(q, K, V, w.dtype, k)                # (also builds and loads the oracle)
        first = time.perf_counter() - t0
        reps = int(min(1000, max(3, 1.0 / max(first, 1e-4))))       # about a second of wall time at least
        t0 = time.perf_counter()
        for _ in range(reps):
            c_oracle.topk_attention(q, K, V, w.dtype, k)
        cpu_s = (time.perf_counter() - t0) / reps
        what = "full decode steps of the same workload" if B == 1 else f"decode steps of one of the {B} sequences"
        cpu = {"value": Hkv * N / cpu_s, "unit": "keys/s", "cores": c_oracle.num_threads(), "kind": "oracle",
               "sample": f"{reps} {what} ({Hq} heads x {N} keys), {cpu_s:.3g} s each "
                         f"({reps * cpu_s * c_oracle.num_threads():.0f} core-seconds)"}

    res = {
        "metric": "kv_keys_scored_per_sec_per_decode_step_N1M" if args.workload == "c3"
        else "kv_keys_scored_per_sec_per_decode_step_" + args.workload,
        "value": keys_per_s,
        "unit": "keys/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {wl.F32: "f32", wl.F16: "f16", wl.BF16: "bf16"}[w.dtype],
        "data": "synthetic",
        "config": {"workload": w.name, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d, "n_tokens": N,
                   "k": k, "layers_rotated": L, "n_seqs": B, "queries_per_step": M,
                   "search": "int8 index + exact refinement" if args.index else
                   (f"page index, bound scale {args.beta:g}" + (" (exact)" if args.beta == 1.0 else " (approximate)")) if args.pages else "exact",
                   **({"pages_read": pages_read, "pages_total": pages_total} if args.pages else {}),
                   **({"sigma": args.sigma or wl.CLUSTER_SIGMA} if args.workload == "c6" else {}),
                   **({"window": args.window} if args.window else {}),
                   **({"forced": "every head redone exactly (worst case of the filtered path)"} if args.force_redo else {})},
        "scores_per_sec": B * M * Hq * N / (ms_per_step * 1e-3),
        "step_hbm_gbps": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_pct_of_hbm_peak": 100.0 * alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "step_ms_gpu_events": ev0.elapsed_time(ev1) / args.steps,
        "step_ms_median": per_step[len(per_step) // 2],
        "step_ms_min": per_step[0],
        "read_probe_gbps": probe_gbps,
        "filter_fallback_heads": fallbacks,
        "roofline": {"bound": "hbm", "kernel": scan_kernel, "achieved": scan_gbps,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": scan_gbps / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(scan_kernel, w.name) if default and M == 1 and not args.index else None, "ms_per_launch": scan_ms,
                     "bytes_per_launch": scan_bytes,
                     "frac_of_read_probe": scan_gbps / probe_gbps},
        "cpu_baseline": cpu,
        "input_generation_s": gen_s,
    }
    print(json.dumps(res))
    cache.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
