"""Seeded random sweep of shapes and entry points against the oracle: dtype, head_dim, head
grouping, cache length (also at and around tile boundaries), k, queries per sequence, causal
visibility, window and pipeline are drawn at random; every case is judged like the
hand-picked ones (index sets exact on margin-enforced inputs; recall for the int8 index).
Two further sweeps draw shapes for the forced redo of every row and for the page index over
clustered caches.
"""
import numpy as np
import pytest
import torch

import helpers as H
from oracle import c_oracle
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl
import test_gpu_index as TI
import test_gpu_multi as TM

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None


def draw_case(rng):
    dtype = int(rng.choice([wl.F16, wl.BF16, wl.F32], p=[0.45, 0.4, 0.15]))
    d = int(rng.choice([32, 64, 128, 256], p=[0.1, 0.3, 0.5, 0.1]))
    G = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 20, 32, 64]))
    if dtype == wl.F32:
        G = min(G, 16)            # fp32 caches: groups up to 16
    Hkv = int(rng.integers(1, 4))
    kind = rng.choice(["tiny", "small", "mid", "big"], p=[0.2, 0.3, 0.3, 0.2])
    N = int({"tiny": rng.integers(1, 200), "small": rng.integers(200, 5000), "mid": rng.integers(5000, 40000),
             "big": rng.integers(40000, 120000)}[kind])
    if rng.random() < 0.25:
        N = max(1, (N // 64) * 64 + int(rng.integers(-1, 2)))
    k = int(rng.integers(1, max(2, min(N + 5, 4000 if N > 20000 else N + 5))))
    if rng.random() < 0.15:
        k = 1
    M = int(rng.choice([1, 1, 1, 2, 3, 4, 5, 7]))
    causal = bool(rng.random() < 0.7)
    if causal and N < M:
        M = 1
    window = min(int(rng.choice([0, 0, 0, 1, 17, 300, N, N + 3])) if rng.random() < 0.4 else 0, 2000)
    use_index = dtype != wl.F32 and d in (64, 128, 256) and G <= 4 and M == 1 and rng.random() < 0.35
    path = ta.PATH_INDEX if use_index else int(rng.choice([ta.PATH_AUTO, ta.PATH_FULL, ta.PATH_FILTER]))
    if M > 1 and N >= 64:
        k = max(1, min(k, N // 8))       # many rows per KV head: keep the margin enforcement convergent
    return dict(dtype=dtype, d=d, Hq=G * Hkv, Hkv=Hkv, N=N, k=k, M=M, causal=causal, window=window, path=path,
                data_seed=int(rng.integers(1 << 30)), slack=int(rng.integers(0, 70)))


def run_drawn(c, label):
    dtype, d, Hq, Hkv, N, k, M, window, path = (c[x] for x in ("dtype", "d", "Hq", "Hkv", "N", "k", "M", "window", "path"))
    """Returns True if the case was judged with an enforced margin (exact sets), False if the margin could
    not be enforced and the case was judged by helpers.check_unmargined."""
    if M > 1:
        q, K, V, delta = TM.make_multi(M, Hq, Hkv, N, d, dtype, k, c["causal"], window, seed=c["data_seed"],
                                       allow_unmargined=True)
        TM.run_multi_case(q, K, V, delta, dtype, k, c["causal"], window, path, label=label)
        return delta is not None
    g = np.random.default_rng(c["data_seed"])
    q = wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), dtype)
    K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    P = max(0, N - window)
    margin_ok = True
    if 0 < k < P:
        Kp = np.ascontiguousarray(K[:, :P])
        try:
            Kp, _, _ = H.enforce_margin(q, Kp, dtype, k)
        except H.MarginNotReached:       # Kp is what the last round left: as good an input as any
            margin_ok = False
        K[:, :P] = Kp
    if path == ta.PATH_INDEX:
        TI.run_index_case(q, K, V, dtype, k, window, label=label, expect_fallbacks=None, margin_ok=margin_ok)
        return margin_ok
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N + c["slack"], k, dtype, max_window=window)
    try:
        cache.set_path(path)
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        res = cache.decode(0, H.to_torch(q, dtype, DEV)[None].contiguous(), k, window=window)
        torch.cuda.synchronize()
        res = tuple(t[0].cpu().numpy() for t in res)
        if margin_ok:
            ref = c_oracle.topk_attention_window(q, K, V, dtype, k, window)
            H.check_against_oracle(*res, ref, H.score_margin(q, K, dtype), min(k, P), H.out_tolerance(dtype),
                                   float(np.abs(wl.widen(V, dtype)).max()), label)
        else:
            H.check_unmargined(res, q, K, V, dtype, k, window, label + " (no margin)")
    finally:
        cache.close()
    return margin_ok


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_and_entry_points(seed):
    rng = np.random.default_rng(seed)
    done = margined = 0
    for i in range(40):
        c = draw_case(rng)
        margined += run_drawn(c, f"sweep seed {seed} case {i} {c}")     # every draw reaches the GPU and the oracle
        done += 1
    print(f"sweep seed {seed}: {done} cases judged, {margined} of them with an enforced margin", flush=True)
    assert done == 40 and margined >= 30


@pytest.mark.parametrize("seed", [21, 22])
def test_random_ragged_batches(seed):
    """Two to four sequences of very different length in one call (a few tokens, a few thousand,
    tens of thousands), a random layer of two (the other holds data of another length), every
    entry point and pipeline; each sequence is judged against the oracle on its own."""
    rng = np.random.default_rng(seed)
    done = 0
    for case in range(25):
        dtype = int(rng.choice([wl.F16, wl.BF16, wl.F32], p=[0.45, 0.4, 0.15]))
        d = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.integers(1, 3))
        Hq = G * Hkv
        B, layer = int(rng.integers(2, 5)), int(rng.integers(0, 2))
        lens = [int(rng.choice([rng.integers(1, 300), rng.integers(300, 9000), rng.integers(33000, 70000)]))
                for _ in range(B)]
        M = int(rng.choice([1, 1, 2, 3]))
        causal = bool(rng.random() < 0.7)
        if causal:
            lens = [max(n, M) for n in lens]
        k = int(rng.integers(1, 600))
        window = int(rng.choice([0, 0, 5, 200]))
        use_index = dtype != wl.F32 and G <= 4 and M == 1 and rng.random() < 0.4
        path = ta.PATH_INDEX if use_index else int(rng.choice([ta.PATH_AUTO, ta.PATH_FULL, ta.PATH_FILTER]))
        sd = int(rng.integers(1 << 30))
        label = f"ragged sweep seed {seed} case {case}: dtype={dtype} d={d} Hq={Hq} Hkv={Hkv} lens={lens} k={k} M={M} " \
                f"causal={causal} window={window} path={path}"
        data = [TM.make_multi(M, Hq, Hkv, n, d, dtype, k, causal, window, seed=sd + b, allow_unmargined=True)
                for b, n in enumerate(lens)]
        cache = ta.TopkAttnCache(2, B, Hq, Hkv, d, max(lens) + 7, k, dtype, max_window=window, max_queries=M,
                                 index_kind=ta.INDEX_INT8 if use_index else ta.INDEX_NONE)
        try:
            cache.set_path(path)
            for b, (q, K, V, delta) in enumerate(data):
                half = max(1, lens[b] // 2)
                cache.append(layer, b, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
                cache.append(1 - layer, b, H.to_torch(V[:, :half].copy(), dtype, DEV),
                             H.to_torch(K[:, :half].copy(), dtype, DEV), head_major=True)
            qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()          # [B, M, Hq, d]
            if M == 1:
                res = cache.decode(layer, qd[:, 0].contiguous(), k, window=window)
            else:
                res = cache.decode_multi(layer, qd, k, causal=causal, window=window)
            torch.cuda.synchronize()
            for b, (q, K, V, delta) in enumerate(data):
                r = tuple(t[b].cpu().numpy() for t in res)
                if M > 1:
                    TM.check_multi(r, q, K, V, dtype, k, causal, window, delta, f"{label} seq {b}")
                elif use_index:
                    TI.check_index_result(r, q[0], K, V, dtype, k, window, f"{label} seq {b}", margin_ok=delta is not None)
                elif delta is None:
                    H.check_unmargined(r, q[0], K, V, dtype, k, window, f"{label} seq {b} (no margin)")
                else:
                    ref = c_oracle.topk_attention_window(q[0], K, V, dtype, k, window)
                    H.check_against_oracle(*r, ref, delta[0], min(k, max(0, lens[b] - window)), H.out_tolerance(dtype),
                                           float(np.abs(wl.widen(V, dtype)).max()), f"{label} seq {b}")
            done += 1
        finally:
            cache.close()
    assert done == 25          # every drawn batch reaches the GPU and the oracle


@pytest.mark.parametrize("seed", [31, 32])
def test_random_shapes_with_every_row_redone(seed):
    """Forced redo (the tail scores every row's keys again and sorts them) over random 16-bit shapes, head
    groups of both scan kernels, chunks of queries, windows; judged against the oracle without a margin."""
    rng = np.random.default_rng(seed)
    for case in range(14):
        dtype = int(rng.choice([wl.F16, wl.BF16]))
        d = int(rng.choice([32, 64, 128, 256], p=[0.1, 0.3, 0.5, 0.1]))
        G = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 20]))
        Hkv = int(rng.integers(1, 3))
        N = int(rng.integers(20000, 200000))
        if rng.random() < 0.3:
            N = (N // 64) * 64 + int(rng.integers(-1, 2))
        k = int(rng.integers(1, 3000))
        M = int(rng.choice([1, 1, 1, 2, 3, 5]))
        causal = bool(rng.integers(0, 2))
        window = int(rng.choice([0, 0, 100, 1000]))
        sd = int(rng.integers(0, 2 ** 31))
        label = f"redo sweep seed {seed} case {case}: dtype={dtype} d={d} G={G} Hkv={Hkv} N={N} k={k} M={M} causal={causal} window={window}"
        print(label, flush=True)
        g = np.random.default_rng(sd)
        Hq = G * Hkv
        q = wl.make_query_chunk(wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), dtype), dtype, M, sd)
        K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
        V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
        cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_window=window, max_queries=M)
        try:
            cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
            ta.topk_attn_debug_force_redo(cache.h, True)
            res = cache.decode_multi(0, H.to_torch(q, dtype, DEV)[None].contiguous(), k, causal=causal, window=window)
            torch.cuda.synchronize()
            TM.check_multi(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, causal, window, None, label)
        finally:
            cache.close()


@pytest.mark.parametrize("seed", [41, 42])
def test_random_clustered_caches_through_the_page_index(seed):
    """Page index over random clustered caches (ragged batches, caches appended in two pieces, windows,
    tight and loose runs): the selection of the plain scan of the same handle, and the oracle's."""
    rng = np.random.default_rng(seed)
    for case in range(14):
        dtype = int(rng.choice([wl.F16, wl.BF16]))
        d = int(rng.choice([32, 64, 128, 256], p=[0.1, 0.3, 0.5, 0.1]))
        G = int(rng.choice([1, 2, 3, 4]))
        Hkv = int(rng.integers(1, 4))
        Hq = G * Hkv
        N = int(rng.integers(300, 150000))
        if rng.random() < 0.3:
            N = max(64, (N // 64) * 64 + int(rng.integers(-1, 2)))
        k = int(rng.integers(1, min(N, 3000) + 1))
        window = int(rng.choice([0, 0, 37, 64, 1000]))
        sigma = float(rng.choice([0.01, 0.03, 0.1, 1.0]))
        lens = [N] + [int(rng.integers(1, N + 1)) for _ in range(int(rng.choice([0, 0, 1, 2])))]
        sd = int(rng.integers(0, 2 ** 31))
        label = f"pages sweep seed {seed} case {case}: dtype={dtype} d={d} G={G} Hkv={Hkv} lens={lens} k={k} window={window} sigma={sigma}"
        print(label, flush=True)
        cache = ta.TopkAttnCache(1, len(lens), Hq, Hkv, d, N, k, dtype, index_kind=ta.INDEX_PAGES, max_window=window)
        try:
            data = []
            for b, n in enumerate(lens):
                w = wl.Workload("sweep", 6, 1, 1, Hq, Hkv, d, n, k, dtype, "clustered")
                q, K, V = (wl.quantize(a, dtype) for a in wl.make_clustered(w, sd + b, sigma, threads=8))
                data.append((q, K, V))
                cut = int(rng.integers(0, n + 1))
                Kd, Vd = H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV)
                if cut > 0:
                    cache.append(0, b, Kd[:, :cut].contiguous(), Vd[:, :cut].contiguous(), head_major=True)
                if cut < n:
                    cache.append(0, b, Kd[:, cut:].contiguous(), Vd[:, cut:].contiguous(), head_major=True)
            qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()
            plain = cache.decode(0, qd, k, window=window)
            cache.set_path(ta.PATH_PAGES)
            res = cache.decode(0, qd, k, window=window)
            torch.cuda.synchronize()
            assert torch.equal(torch.sort(res[1], dim=2).values, torch.sort(plain[1], dim=2).values), label
            np.testing.assert_allclose(res[0].cpu().numpy(), plain[0].cpu().numpy(), rtol=3e-5, atol=2e-6, err_msg=label)
            for b in range(len(lens)):
                q, K, V = data[b]
                H.check_unmargined(tuple(t[b].cpu().numpy() for t in res), q, K, V, dtype, k, window, f"{label} seq {b}")
        finally:
            cache.close()
