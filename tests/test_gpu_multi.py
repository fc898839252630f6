"""GPU parity for the row-tile scan: head groups of 5..16 on the filtered path, and chunks
of M queries per sequence (topk_attn_decode_multi), against the CPU oracle through the
C ABI.  Same bars as test_gpu_parity.py.
"""
import numpy as np
import pytest
import torch

import helpers as H
from oracle import c_oracle
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl
from test_gpu_parity import rand_case, run_case

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None


# ------------------------------------------------------------------ wide head groups, one query
@pytest.mark.parametrize("dtype,Hq,Hkv,N,d,k,path", [
    (wl.F16, 16, 2, 40000, 128, 300, ta.PATH_AUTO),      # G = 8
    (wl.BF16, 16, 1, 33001, 64, 500, ta.PATH_AUTO),      # G = 16: a full row tile
    (wl.F16, 10, 2, 36001, 128, 64, ta.PATH_AUTO),       # G = 5: rows 5..15 of the tile unused
    (wl.BF16, 24, 2, 70001, 128, 1, ta.PATH_AUTO),       # G = 12, k = 1
    (wl.F16, 14, 2, 4097, 64, 130, ta.PATH_FULL),        # G = 7, all scores stored
    (wl.F16, 16, 2, 3000, 128, 200, ta.PATH_FILTER),     # short cache forced through the filter
    (wl.BF16, 64, 2, 36000, 128, 100, ta.PATH_AUTO),     # G = 32: one block of two row tiles per KV head
    (wl.F16, 48, 1, 40001, 64, 50, ta.PATH_AUTO),        # multi-query attention, 48 heads on one KV head: two blocks
    (wl.F16, 40, 1, 2000, 128, 30, ta.PATH_FULL),        # G = 40, all scores stored
    (wl.F16, 16, 2, 40000, 128, 14000, ta.PATH_FILTER),  # G = 8, a third of the keys selected
])
def test_wide_head_groups(dtype, Hq, Hkv, N, d, k, path):
    q, K, V = rand_case(Hq, Hkv, N, d, dtype, k, seed=N + k)
    run_case(q, K, V, dtype, k, path=path, chunks=2, label=f"G={Hq // Hkv} N={N} k={k}",
             expect_fallbacks=0 if path == ta.PATH_AUTO else None)


# ------------------------------------------------------------------ several queries per sequence
def make_multi(M, Hq, Hkv, N, d, dtype, k, causal, window, seed, allow_unmargined=False):
    """delta is None when `allow_unmargined` and the margin could not be enforced (the keys are then
    whatever the last round left, as good an input as any; check_multi judges it without a margin)."""
    g = np.random.default_rng(seed)
    q0 = wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), dtype)
    q = wl.make_query_chunk(q0, dtype, M, seed)
    K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    try:
        K, delta = H.enforce_margin_multi(q, K, dtype, k, causal, window)
    except H.MarginNotReached:
        if not allow_unmargined:
            raise
        delta = None
    return q, K, V, delta


def check_multi(res, q, K, V, dtype, k, causal, window, delta, label):
    """res = (out, idx, vals, lse) numpy arrays [M, Hq, ...] of one sequence."""
    M, Hq, d = q.shape
    N = K.shape[1]
    if delta is None:           # no margin on these inputs: every query is judged on its own visible part
        for m in range(M):
            n_vis = N - (M - 1 - m) if causal else N
            H.check_unmargined(tuple(r[m] for r in res), q[m], np.ascontiguousarray(K[:, :n_vis]),
                               np.ascontiguousarray(V[:, :n_vis]), dtype, k, window, f"{label} query {m} (no margin)")
        return
    ref = c_oracle.topk_attention_multi(q, K, V, dtype, k, causal, window)
    vmax = float(np.abs(wl.widen(V, dtype)).max())
    for m in range(M):
        n_vis = N - (M - 1 - m) if causal else N
        k_eff = min(k, n_vis - min(window, n_vis))
        H.check_against_oracle(res[0][m], res[1][m], res[2][m], res[3][m], tuple(r[m] for r in ref), delta[m],
                               k_eff, H.out_tolerance(dtype), vmax, f"{label} query {m}")


def run_multi_case(q, K, V, delta, dtype, k, causal, window=0, path=ta.PATH_AUTO, label="", expect_fallbacks=None):
    M, Hq, d = q.shape
    Hkv, N, _ = K.shape
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_window=window, max_queries=M)
    try:
        cache.set_path(path)
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        out, idx, vals, lse = cache.decode_multi(0, qd, k, causal=causal, window=window)
        torch.cuda.synchronize()
        fb = cache.last_fallbacks()
        check_multi(tuple(t[0].cpu().numpy() for t in (out, idx, vals, lse)), q, K, V, dtype, k, causal, window,
                    delta, label)
        if expect_fallbacks is not None:
            assert fb == expect_fallbacks, f"{label}: {fb} rows fell back"
    finally:
        cache.close()


@pytest.mark.parametrize("dtype,M,Hq,Hkv,N,d,k,causal,window,path", [
    (wl.F16, 4, 8, 2, 36000, 128, 300, True, 0, ta.PATH_AUTO),      # 4 queries x 4 heads: one full row tile
    (wl.BF16, 3, 8, 2, 50001, 64, 1000, False, 0, ta.PATH_AUTO),    # 12 rows, every query sees everything
    (wl.F16, 7, 8, 2, 35000, 128, 200, True, 100, ta.PATH_AUTO),    # two row blocks (4 + 3 queries), window
    (wl.F16, 5, 16, 2, 34000, 128, 128, True, 0, ta.PATH_AUTO),     # G = 8: blocks of 2, 2, 1 queries
    (wl.BF16, 2, 16, 1, 33000, 64, 77, True, 0, ta.PATH_AUTO),      # G = 16: one query per block
    (wl.F16, 6, 6, 2, 18000, 128, 90, True, 0, ta.PATH_FILTER),     # G = 3: blocks of 5 and 1 queries
    (wl.F16, 4, 4, 1, 700, 128, 60, True, 0, ta.PATH_FULL),         # all scores stored, row-tile kernel
    (wl.F32, 3, 4, 2, 3000, 64, 50, True, 0, ta.PATH_AUTO),         # fp32: plain-FMA scorer per query
    (wl.F16, 16, 2, 2, 34000, 128, 150, True, 0, ta.PATH_AUTO),     # MQA-like: 16 queries x 1 head
    (wl.F16, 3, 16, 2, 36000, 256, 100, True, 0, ta.PATH_AUTO),     # d = 256, G = 8: 24 rows in two row tiles
    (wl.BF16, 2, 8, 2, 40000, 256, 300, False, 50, ta.PATH_AUTO),   # d = 256, 8 rows, window
    (wl.F16, 5, 8, 2, 35000, 32, 120, True, 0, ta.PATH_AUTO),       # d = 32, 20 rows
    (wl.F16, 3, 20, 1, 36000, 128, 64, True, 0, ta.PATH_AUTO),      # G = 20, 60 rows: blocks cut across queries
    (wl.F16, 33, 4, 1, 33500, 64, 100, True, 16, ta.PATH_AUTO),     # 9 row blocks, the last with one query
    (wl.F16, 3, 8, 2, 36000, 128, 9000, True, 0, ta.PATH_FILTER),   # a quarter of the keys selected: the per-row
    (wl.BF16, 6, 8, 2, 34000, 64, 12000, True, 0, ta.PATH_FILTER),  # stages flush every few tiles (12 and 24 rows)
])
def test_multi_query_decode(dtype, M, Hq, Hkv, N, d, k, causal, window, path):
    q, K, V, delta = make_multi(M, Hq, Hkv, N, d, dtype, k, causal, window, seed=N + k + M)
    run_multi_case(q, K, V, delta, dtype, k, causal, window, path,
                   label=f"multi M={M} G={Hq // Hkv} N={N} k={k}",
                   expect_fallbacks=0 if path == ta.PATH_AUTO and dtype != wl.F32 else None)


def test_multi_short_cache_edges():
    """k beyond the visible length, a window that swallows the whole visible part of the
    first queries, and a cache exactly as long as the chunk."""
    dtype, M, Hq, Hkv, d = wl.F16, 4, 4, 2, 64
    for N, k, window in [(5, 10, 2), (4, 3, 0), (9, 2, 7), (130, 64, 1)]:
        q, K, V, delta = make_multi(M, Hq, Hkv, N, d, dtype, k, True, window, seed=N)
        for path in (ta.PATH_FULL, ta.PATH_FILTER):
            run_multi_case(q, K, V, delta, dtype, k, True, window, path, label=f"edge N={N} k={k} W={window}")


def test_multi_batch_ragged_and_single_query_equivalence():
    """Two sequences of different length decoded together with M = 3; each query's result
    must also be what a plain decode of a cache truncated to its visible length returns
    (bit for bit in idx order-insensitive form), and n_queries = 1 is the plain decode."""
    dtype, M, Hq, Hkv, d, k = wl.BF16, 3, 8, 2, 128, 200
    lens = [36000, 33003]
    cache = ta.TopkAttnCache(1, 2, Hq, Hkv, d, max(lens), k, dtype, max_queries=M)
    try:
        data = []
        for b, n in enumerate(lens):
            q, K, V, delta = make_multi(M, Hq, Hkv, n, d, dtype, k, True, 0, seed=70 + b)
            data.append((q, K, V, delta))
            cache.append(0, b, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()      # [B, M, Hq, d]
        out, idx, vals, lse = cache.decode_multi(0, qd, k, causal=True)
        torch.cuda.synchronize()
        assert cache.last_fallbacks() == 0
        for b in range(2):
            q, K, V, delta = data[b]
            check_multi(tuple(t[b].cpu().numpy() for t in (out, idx, vals, lse)), q, K, V, dtype, k, True, 0, delta,
                        f"ragged seq {b}")
        # the last query of each chunk sees the whole cache: same as the plain decode of that query
        out1, idx1, vals1, lse1 = cache.decode(0, qd[:, M - 1].contiguous(), k)
        torch.cuda.synchronize()
        assert torch.equal(torch.sort(idx1, dim=-1).values, torch.sort(idx[:, M - 1], dim=-1).values)
        np.testing.assert_allclose(out1.cpu().numpy(), out[:, M - 1].cpu().numpy(), rtol=1e-5, atol=1e-6)
        # n_queries = 1 through the multi entry point is the plain decode, bit for bit
        o2 = torch.empty_like(out1)
        i2 = torch.empty_like(idx1)
        st = torch.cuda.current_stream().cuda_stream
        q_last = qd[:, M - 1].contiguous()
        ta.topk_attn_decode_multi(cache.h, 0, q_last.data_ptr(), 1, True, k, 0, o2.data_ptr(), i2.data_ptr(), 0, 0, st)
        torch.cuda.synchronize()
        assert torch.equal(o2, out1) and torch.equal(i2, idx1)
    finally:
        cache.close()


def test_multi_repeatable_and_error_codes():
    dtype, M, Hq, Hkv, d, N, k = wl.F16, 4, 8, 2, 128, 20000, 100
    q, K, V, delta = make_multi(M, Hq, Hkv, N, d, dtype, k, True, 0, seed=5)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_queries=M)
    try:
        L = ta.lib()
        st = torch.cuda.current_stream().cuda_stream
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        o = torch.empty((1, M, Hq, d), dtype=torch.float32, device=DEV)
        # fewer cached tokens than queries in a causal chunk
        cache.append(0, 0, H.to_torch(K[:, :3].copy(), dtype, DEV), H.to_torch(V[:, :3].copy(), dtype, DEV),
                     head_major=True)
        assert L.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), M, 1, k, 0, o.data_ptr(), None, None, None, st) == ta.EINVAL
        assert L.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), M, 0, k, 0, o.data_ptr(), None, None, None, st) == ta.OK
        cache.append(0, 0, H.to_torch(K[:, 3:].copy(), dtype, DEV), H.to_torch(V[:, 3:].copy(), dtype, DEV),
                     head_major=True)
        assert L.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), M + 1, 1, k, 0, o.data_ptr(), None, None, None, st) == ta.EINVAL
        assert L.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), 0, 1, k, 0, o.data_ptr(), None, None, None, st) == ta.EINVAL
        assert L.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), M, 1, k, 1, o.data_ptr(), None, None, None, st) == ta.EINVAL   # max_window 0
        a = cache.decode_multi(0, qd, k, causal=True)
        b = cache.decode_multi(0, qd, k, causal=True)
        torch.cuda.synchronize()
        for x, y in zip(a, b):
            assert torch.equal(x, y)
        check_multi(tuple(t[0].cpu().numpy() for t in a), q, K, V, dtype, k, True, 0, delta, "repeat")
    finally:
        cache.close()


def test_c3_chunk_of_four_queries_1m_fp16():
    """The N = 1M configuration (32 query heads, 8 KV heads, d = 128, fp16, k = 16384) with
    a causal chunk of four queries: one full 16-row tile per KV head."""
    w = wl.C3
    M = 4
    q0, K, V = wl.make_quantized(w, 0, threads=16)
    q = wl.make_query_chunk(q0, w.dtype, M, 11)
    K, delta = H.enforce_margin_multi(q, K, w.dtype, w.k, True, 0, shrink=2.0 ** -9)   # 16 rows per KV head
    run_multi_case(q, K, V, delta, w.dtype, w.k, True, 0, ta.PATH_AUTO, label="c3 x4", expect_fallbacks=0)


def test_multi_batched_wide_groups_ragged():
    """Three sequences of different length, head groups of 8, three queries each (row blocks
    of two and one query), causal with a window."""
    dtype, M, Hq, Hkv, d, k, W = wl.F16, 3, 16, 2, 64, 120, 50
    lens = [34000, 300, 33001]          # the middle one takes the exact general path with the others
    cache = ta.TopkAttnCache(1, 3, Hq, Hkv, d, max(lens), k, dtype, max_window=W, max_queries=M)
    try:
        data = []
        for b, n in enumerate(lens):
            q, K, V, delta = make_multi(M, Hq, Hkv, n, d, dtype, k, True, W, seed=80 + b)
            data.append((q, K, V, delta))
            cache.append(0, b, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()
        res = cache.decode_multi(0, qd, k, causal=True, window=W)
        torch.cuda.synchronize()
        for b in range(3):
            q, K, V, delta = data[b]
            check_multi(tuple(t[b].cpu().numpy() for t in res), q, K, V, dtype, k, True, W, delta, f"wide ragged seq {b}")
    finally:
        cache.close()


@pytest.mark.parametrize("dtype,M,Hq,Hkv,N,d,k,causal,window", [
    (wl.F16, 4, 8, 2, 200000, 128, 700, True, 0),
    (wl.BF16, 3, 16, 2, 150000, 64, 400, True, 64),      # G = 8, a window beside the search
    (wl.F16, 9, 4, 1, 120000, 128, 300, False, 0),       # three row blocks
])
def test_multi_every_row_sorted_again(dtype, M, Hq, Hkv, N, d, k, causal, window):
    """Forced redo of a chunk of queries: the tail scores every row's keys again (each query over its own
    visible prefix) and must keep exactly what the row-tile scan counted; then the same call unforced."""
    q, K, V, delta = make_multi(M, Hq, Hkv, N, d, dtype, k, causal, window, seed=N + M, allow_unmargined=True)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_window=window, max_queries=M)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        ta.topk_attn_debug_force_redo(cache.h, True)
        res = cache.decode_multi(0, qd, k, causal=causal, window=window)
        torch.cuda.synchronize()
        rec = ta.topk_attn_last_selection_records(cache.h, M * Hq)
        dims = ta.topk_attn_debug_read_workspace_dims(cache.h)
        kept = ta.topk_attn_debug_read_workspace(cache.h, "seg_cnt2", np.uint32, dims[4] * M * Hq).reshape(M * Hq, dims[4])
        for r in range(M * Hq):
            assert rec[r][0] >> 8 == 4 and rec[r][0] & 0xFF == 0, f"row {r}: record {rec[r]}"   # forced, sorted again, not dense
            assert kept[r].sum() == rec[r][1] + rec[r][3], f"row {r}: kept {kept[r].sum()}, counted {rec[r][1]} + {rec[r][3]}"
        check_multi(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, causal, window, delta, "forced redo of a chunk")
        ta.topk_attn_debug_force_redo(cache.h, False)
        res2 = cache.decode_multi(0, qd, k, causal=causal, window=window)
        torch.cuda.synchronize()
        assert torch.equal(torch.sort(res2[1], dim=-1).values, torch.sort(res[1], dim=-1).values)
        np.testing.assert_allclose(res2[0].cpu().numpy(), res[0].cpu().numpy(), rtol=2e-5, atol=1e-6)
    finally:
        cache.close()


def test_other_entry_points_under_graph_capture_replays():
    """A chunk of queries (row-tile scan), the int8 index and the entry point that allocates nothing, each
    captured in a HIP graph and replayed with eager work in between: every replay equals the eager call on the
    same inputs (the eager results are judged against the oracle by the other tests)."""
    dtype, Hq, Hkv, d, N, k, M, W = wl.F16, 8, 2, 128, 60000, 400, 3, 200
    g0 = np.random.default_rng(909)
    K = wl.quantize(g0.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    V = wl.quantize(g0.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    qs = [wl.make_query_chunk(wl.quantize(g0.standard_normal((Hq, d)).astype(np.float32), dtype), dtype, M, 5 + i) for i in range(2)]
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_window=W, max_queries=M, index_kind=ta.INDEX_INT8)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(qs[0], dtype, DEV)[None].contiguous()                 # [1, M, Hq, d]
        q1 = qd[:, 0].contiguous()                                            # one query per sequence
        out = torch.empty((1, M, Hq, d), dtype=torch.float32, device=DEV)
        idx = torch.empty((1, M, Hq, k), dtype=torch.int32, device=DEV)
        vals = torch.empty((1, M, Hq, k), dtype=torch.float32, device=DEV)
        lse = torch.empty((1, M, Hq), dtype=torch.float32, device=DEV)
        ptrs = (out.data_ptr(), idx.data_ptr(), vals.data_ptr(), lse.data_ptr())
        s = torch.cuda.Stream()
        calls = {
            "chunk": (lambda: ta.topk_attn_decode_multi(cache.h, 0, qd.data_ptr(), M, True, k, W, *ptrs, s.cuda_stream),
                      lambda: cache.decode_multi(0, qd, k, causal=True, window=W), ta.PATH_AUTO, M),
            "index": (lambda: ta.topk_attn_decode_window(cache.h, 0, q1.data_ptr(), k, W, *ptrs, s.cuda_stream),
                      lambda: cache.decode(0, q1, k, window=W), ta.PATH_INDEX, 1),
            "static": (lambda: ta.topk_attn_decode_static(cache.h, 0, q1.data_ptr(), k, *ptrs, s.cuda_stream),
                       lambda: cache.decode(0, q1, k), ta.PATH_AUTO, 1),
        }
        with torch.cuda.stream(s):
            for name, (raw_call, eager_call, path, m) in calls.items():
                cache.set_path(path)
                raw_call()                                                     # warm-up outside the capture
                s.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=s):
                    raw_call()
                for rep, q in enumerate([qs[0], qs[1], qs[0]]):
                    qd.copy_(H.to_torch(q, dtype, DEV)[None])                  # eager work between replays
                    q1.copy_(qd[:, 0])
                    out.zero_(); idx.zero_(); lse.zero_()
                    s.synchronize()
                    g.replay()
                    s.synchronize()
                    got = (out.clone(), idx.clone(), lse.clone())
                    eager = eager_call()
                    s.synchronize()
                    flat = lambda t, n: t.reshape(-1)[:n]
                    n_o, n_i, n_l = m * Hq * d, m * Hq * k, m * Hq
                    assert torch.equal(flat(eager[0], n_o), flat(got[0], n_o)), f"{name} replay {rep}: out"
                    assert torch.equal(flat(eager[1], n_i), flat(got[1], n_i)), f"{name} replay {rep}: idx"
                    assert torch.equal(flat(eager[3], n_l), flat(got[2], n_l)), f"{name} replay {rep}: lse"
    finally:
        cache.close()
