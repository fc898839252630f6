"""GPU tests of the coarse page index (TOPK_ATTN_INDEX_PAGES / TOPK_ATTN_PATH_PAGES), the sub-linear search.

* Index contents: every page's ball (centre, radius) encloses the page's keys and is about as tight
  as the ball around the mean that oracle/page_index_ref.py computes, after appends in pieces.
* The search is exact: index sets, vals, out, lse judged against the exact oracle like the plain
  path, and the same selection as the plain path on the same handle; the pages read include every page
  that holds a selected key (oracle) and, on a cache with topical runs, are a fraction of the cache.
* With a shrunk bound the search is approximate: recall@k against the exact oracle.
"""
import numpy as np
import pytest
import torch

import helpers as H
from oracle import c_oracle
from oracle import int8_index_ref as i8
from oracle import page_index_ref as pg
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None
PAGE = 64


def page_views(cache, L, B, Hkv, Ncap, d, dtype):
    """Centres [L, B, Hkv, P, d] (storage dtype) and balls [L, B, Hkv, P, 2] fp32 as laid out behind K and V."""
    up = lambda x: (x + 255) // 256 * 256
    P = (Ncap + PAGE - 1) // PAGE
    half = up(L * B * Hkv * Ncap * d * 2)
    nc = L * B * Hkv * P * d * 2
    tdt = torch.bfloat16 if dtype == wl.BF16 else torch.float16
    centres = cache.kv[2 * half: 2 * half + nc].view(tdt).view(L, B, Hkv, P, d)
    off = 2 * half + up(nc)
    balls = cache.kv[off: off + L * B * Hkv * P * 8].view(torch.float32).view(L, B, Hkv, P, 2)
    return centres, balls


def clustered(N, k, seed, sigma, dtype=wl.F16, Hq=8, Hkv=2, d=128):
    w = wl.Workload("clustered_test", 6, 1, 1, Hq, Hkv, d, N, k, dtype, "clustered")
    q, K, V = wl.make_clustered(w, seed, sigma, threads=8)
    return wl.quantize(q, dtype), wl.quantize(K, dtype), wl.quantize(V, dtype)


@pytest.mark.parametrize("dtype,d", [(wl.F16, 128), (wl.BF16, 64), (wl.BF16, 256), (wl.F16, 32)])
def test_page_balls_enclose_their_pages_after_piecewise_appends(dtype, d):
    g = np.random.default_rng(d + dtype)
    L, B, Hq, Hkv, Ncap, N = 2, 2, 4, 2, 1000, 903
    K = (g.standard_normal((Hkv, N, d)) * g.uniform(0.05, 4.0, (Hkv, N, 1))).astype(np.float32)
    K[0, 128:192] = K[0, 128]                                  # page 2 of KV head 0: 64 identical keys
    Ks = wl.quantize(K, dtype)
    Vs = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    cache = ta.TopkAttnCache(L, B, Hq, Hkv, d, Ncap, 16, dtype, index_kind=ta.INDEX_PAGES)
    try:
        Kd, Vd = H.to_torch(Ks, dtype, DEV), H.to_torch(Vs, dtype, DEV)
        # layer 1, sequence 1: a bulk import that ends inside a page, single tokens across a page boundary
        # (token-major), then the rest; layer 0 through the batched per-step append
        cache.append(1, 1, Kd[:, :100].contiguous(), Vd[:, :100].contiguous(), head_major=True)
        for t in range(100, 131):
            cache.append(1, 1, Kd[:, t:t + 1].permute(1, 0, 2).contiguous(), Vd[:, t:t + 1].permute(1, 0, 2).contiguous())
        cache.append(1, 1, Kd[:, 131:].contiguous(), Vd[:, 131:].contiguous(), head_major=True)
        cache.append(0, 0, Kd[:, :70].contiguous(), Vd[:, :70].contiguous(), head_major=True)
        cache.append(0, 1, Kd[:, :5].contiguous(), Vd[:, :5].contiguous(), head_major=True)
        steps = [(200, 203), (203, 264), (264, 334)]           # every sequence of layer 0 grows by the same tokens
        for a, z in steps:
            kn = Kd[:, a:z].permute(1, 0, 2)[None].expand(B, -1, -1, -1).contiguous()
            cache.append_step(0, kn, kn.clone())
        torch.cuda.synchronize()
        centres, balls = page_views(cache, L, B, Hkv, Ncap, d, dtype)
        Kw = wl.widen(Ks, dtype)

        def judge(c_dev, b_dev, rows, label):
            P = (rows.shape[1] + PAGE - 1) // PAGE
            c = c_dev[:, :P].float().cpu().numpy().astype(np.float64)
            r = b_dev[:, :P, 0].cpu().numpy().astype(np.float64)
            cn = b_dev[:, :P, 1].cpu().numpy().astype(np.float64)
            slack = pg.ball_slack(rows, PAGE, c, r)
            assert (slack >= 0).all(), f"{label}: a key lies outside its page's ball"
            c_ref, r_ref = pg.page_balls(rows, PAGE)
            # the stored centre is the mean rounded to the storage type: the radius grows by at most that rounding
            step = (2.0 ** -8 if dtype == wl.BF16 else 2.0 ** -11) * np.abs(c_ref).max(axis=2) * np.sqrt(d)
            assert (r <= r_ref * 1.001 + step + 1e-6).all(), f"{label}: radius looser than the ball around the mean"
            assert (cn >= np.sqrt((c ** 2).sum(axis=2)) * (1 - 1e-6)).all() and (cn <= np.sqrt((c ** 2).sum(axis=2)) * 1.001 + 1e-30).all()
            return r

        r = judge(centres[1, 1], balls[1, 1], Kw, "layer 1")
        assert r[0, 2] <= 1e-20 and r[1, 2] > 1e-3              # identical keys: the centre is the key, the radius nothing
        grown = np.concatenate([Kw[:, :70], Kw[:, 200:203], Kw[:, 203:264], Kw[:, 264:334]], axis=1)
        judge(centres[0, 0], balls[0, 0], grown, "layer 0 seq 0")
        grown1 = np.concatenate([Kw[:, :5], Kw[:, 200:203], Kw[:, 203:264], Kw[:, 264:334]], axis=1)
        judge(centres[0, 1], balls[0, 1], grown1, "layer 0 seq 1")
    finally:
        cache.close()


def run_pages_case(q, K, V, dtype, k, beta=1.0, label="", margin=True):
    """One sequence through the page index and through the plain scan of the same handle.  Returns
    (fraction of pages read, recalls per head)."""
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    if margin:
        try:      # a nudge of several ulps of the storage type
            K, _, _ = H.enforce_margin(q, K, dtype, k, shrink=2.0 ** -9 if dtype == wl.F16 else 2.0 ** -6)
        except H.MarginNotReached:
            margin = False
    ref = c_oracle.topk_attention(q, K, V, dtype, k)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, index_kind=ta.INDEX_PAGES)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        plain = cache.decode(0, qd, k)
        plain_fallbacks = cache.last_fallbacks()
        assert ta.topk_attn_last_pages_read(cache.h)[0] == ta.topk_attn_last_pages_read(cache.h)[1]
        cache.set_path(ta.PATH_PAGES)
        if beta != 1.0:
            ta.topk_attn_set_page_bound_scale(cache.h, beta)
        res = cache.decode(0, qd, k)
        torch.cuda.synchronize()
        read, total = ta.topk_attn_last_pages_read(cache.h)
        assert total == Hkv * ((N + PAGE - 1) // PAGE) and 0 < read <= total
        out, idx, vals, lse = (t[0].cpu().numpy() for t in res)
        delta = H.score_margin(q, K, dtype)
        vmax = float(np.abs(wl.widen(V, dtype)).max())
        k_eff = min(k, N)
        recalls = [i8.recall_at_k(idx[h, :k_eff], ref[1][h, :k_eff]) for h in range(Hq)]
        if beta == 1.0:
            assert cache.last_fallbacks() == plain_fallbacks       # same candidates, same lists
            if margin:
                H.check_against_oracle(out, idx, vals, lse, ref, delta, k_eff, H.out_tolerance(dtype), vmax, label)
            else:
                H.check_unmargined((out, idx, vals, lse), q, K, V, dtype, k, 0, label)
            # same candidates as the plain scan: the same selection; the pages kept are dealt to the waves in
            # another order than the tiles of the plain scan, so the fp32 sums may differ in their last bits
            assert torch.equal(torch.sort(res[1], dim=2).values, torch.sort(plain[1], dim=2).values), f"{label}: index sets differ from the plain scan's"
            assert torch.equal(torch.sort(res[2], dim=2).values, torch.sort(plain[2], dim=2).values), f"{label}: vals differ from the plain scan's"
            np.testing.assert_allclose(res[0].cpu().numpy(), plain[0].cpu().numpy(), rtol=2e-5, atol=1e-6, err_msg=label)
            np.testing.assert_allclose(res[3].cpu().numpy(), plain[3].cpu().numpy(), rtol=1e-6, err_msg=label)
            again = cache.decode(0, qd, k)                      # and the same bits every time
            torch.cuda.synchronize()
            assert all(torch.equal(a, b) for a, b in zip(again, res)), f"{label}: two runs differ"
            # no page that holds a selected key was skipped: at least those pages were read
            need = pg.pages_holding_topk(ref[1], (N + PAGE - 1) // PAGE, PAGE, G)
            assert read >= need.sum(), f"{label}: fewer pages read than hold selected keys"
        else:
            S = c_oracle.scores(q, K, dtype)
            for h in range(Hq):        # whatever is returned is a valid position with its exact score
                got = idx[h, :k_eff].astype(np.int64)
                assert np.unique(got).size == k_eff and got.min() >= 0 and got.max() < N
                assert np.abs(vals[h, :k_eff].astype(np.float64) - S[h, got]).max() <= delta[h] / 8
        return read / total, recalls
    finally:
        cache.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,N,d,k,sigma", [
    (wl.F16, 8, 2, 70001, 128, 700, 0.02),
    (wl.BF16, 8, 2, 65536, 128, 1024, 0.05),
    (wl.F16, 4, 2, 50003, 64, 300, 0.03),        # G = 2, d = 64
    (wl.BF16, 3, 3, 40000, 256, 500, 0.02),      # G = 1, d = 256
    (wl.F16, 4, 1, 300001, 128, 3000, 0.02),     # one KV head: 1024 wave segments
])
def test_pages_path_is_exact_on_clustered_caches(dtype, Hq, Hkv, N, d, k, sigma):
    q, K, V = clustered(N, k, seed=N + k, sigma=sigma, dtype=dtype, Hq=Hq, Hkv=Hkv, d=d)
    frac, _ = run_pages_case(q, K, V, dtype, k, label=f"pages N={N} k={k} sigma={sigma}")
    print(f"pages N={N} k={k} sigma={sigma}: {frac:.3f} of the pages read", flush=True)
    assert frac < 0.6          # runs this tight leave a good part of the cache unread


def test_pages_path_on_unstructured_keys_reads_everything_and_stays_exact():
    g = np.random.default_rng(8)
    Hq, Hkv, N, d, k = 8, 2, 40001, 128, 300
    q = wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), wl.F16)
    K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), wl.F16)
    V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), wl.F16)
    frac, _ = run_pages_case(q, K, V, wl.F16, k, label="pages gaussian")
    assert frac > 0.99         # Gaussian rows: no page can be ruled out


def test_shrunk_page_bound_trades_recall_for_pages():
    N, k, sigma = 131072, 2048, 0.1
    q, K, V = clustered(N, k, seed=17, sigma=sigma)
    fracs, recs = [], []
    for beta in (1.0, 0.5, 0.1):
        frac, recalls = run_pages_case(q, K, V, wl.F16, k, beta=beta, label=f"beta {beta}", margin=False)
        fracs.append(frac)
        recs.append(min(recalls))
        print(f"beta {beta}: {frac:.3f} of the pages read, recall@k {min(recalls):.4f} .. {max(recalls):.4f}", flush=True)
    assert recs[0] == 1.0
    assert fracs[0] > fracs[1] > fracs[2]
    assert recs[1] >= 0.9 and recs[2] >= 0.3          # a shrunk bound misses keys, the more the smaller it is


def test_pages_ragged_batch_and_windows():
    dtype, Hq, Hkv, d, k = wl.F16, 8, 2, 128, 200
    lens = [60000, 130, 33000]
    cache = ta.TopkAttnCache(1, 3, Hq, Hkv, d, max(lens), k, dtype, index_kind=ta.INDEX_PAGES, max_window=64)
    try:
        cache.set_path(ta.PATH_PAGES)
        data = []
        for b, n in enumerate(lens):
            q, K, V = clustered(n, k, seed=300 + b, sigma=0.03)
            K, _, _ = H.enforce_margin(q, K, dtype, k, shrink=2.0 ** -9)
            data.append((q, K, V))
            cache.append(0, b, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()
        out, idx, vals, lse = cache.decode(0, qd, k)
        torch.cuda.synchronize()
        read, total = ta.topk_attn_last_pages_read(cache.h)
        assert read < total
        for b, n in enumerate(lens):
            q, K, V = data[b]
            ref = c_oracle.topk_attention(q, K, V, dtype, k)
            H.check_against_oracle(out[b].cpu().numpy(), idx[b].cpu().numpy(), vals[b].cpu().numpy(), lse[b].cpu().numpy(),
                                   ref, H.score_margin(q, K, dtype), min(k, n), 2e-3, float(np.abs(wl.widen(V, dtype)).max()),
                                   f"pages ragged seq {b}")
        # with a window the search covers the pages of each sequence's prefix (the last one cut short by the window)
        for window in (64, 37):
            outw, idxw, valsw, lsew = cache.decode(0, qd, k, window=window)
            torch.cuda.synchronize()
            read, total = ta.topk_attn_last_pages_read(cache.h)
            assert read < total
            for b in range(len(lens)):
                q, K, V = data[b]
                H.check_unmargined(tuple(t[b].cpu().numpy() for t in (outw, idxw, valsw, lsew)), q, K, V, dtype, k, window,
                                   f"pages + window {window}, seq {b}")
        assert ta.lib().topk_attn_set_page_bound_scale(cache.h, 0.0) == ta.EINVAL
        assert ta.lib().topk_attn_set_page_bound_scale(cache.h, 1.5) == ta.EINVAL
    finally:
        cache.close()
    plain = ta.TopkAttnCache(1, 1, Hq, Hkv, d, 1000, k, dtype)
    try:
        assert ta.lib().topk_attn_set_path(plain.h, ta.PATH_PAGES) == ta.EINVAL
        assert ta.lib().topk_attn_set_page_bound_scale(plain.h, 0.5) == ta.EINVAL
    finally:
        plain.close()


@pytest.mark.parametrize("dtype,N,d,k,window", [(wl.F16, 300000, 128, 2000, 1000), (wl.BF16, 150001, 64, 700, 4096)])
def test_pages_with_a_window_match_the_plain_scan(dtype, N, d, k, window):
    """Page index and recent-token window together: the search runs over the pages of the prefix before the
    window (its last page cut short by the window), the window's tokens are always attended to."""
    Hq, Hkv = 8, 2
    q, K, V = clustered(N, k, seed=N + window, sigma=0.03, dtype=dtype, Hq=Hq, Hkv=Hkv, d=d)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, index_kind=ta.INDEX_PAGES, max_window=window)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        plain = cache.decode(0, qd, k, window=window)
        cache.set_path(ta.PATH_PAGES)
        res = cache.decode(0, qd, k, window=window)
        torch.cuda.synchronize()
        read, total = ta.topk_attn_last_pages_read(cache.h)
        print(f"pages + window: {read} of {total} pages read", flush=True)
        assert 0 < read < 0.7 * total
        H.check_unmargined(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, window, "pages + window")
        assert torch.equal(torch.sort(res[1], dim=2).values, torch.sort(plain[1], dim=2).values)
        np.testing.assert_allclose(res[0].cpu().numpy(), plain[0].cpu().numpy(), rtol=2e-5, atol=1e-6)
        np.testing.assert_allclose(res[3].cpu().numpy(), plain[3].cpu().numpy(), rtol=1e-6)
    finally:
        cache.close()


def test_page_index_decode_under_graph_capture_replays():
    """A decode through the page index with a window, captured in a HIP graph (page filter, page list, paged
    scan, tail: kernels only) and replayed with eager work in between: every replay gives the eager result,
    also after the query has changed (another set of pages is kept)."""
    dtype, Hq, Hkv, d, N, k, W = wl.F16, 8, 2, 128, 120000, 900, 300
    q1, K, V = clustered(N, k, seed=77, sigma=0.03, dtype=dtype, Hq=Hq, Hkv=Hkv, d=d)
    q2 = wl.quantize(np.random.default_rng(78).standard_normal((Hq, d)).astype(np.float32), dtype)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, index_kind=ta.INDEX_PAGES, max_window=W)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        cache.set_path(ta.PATH_PAGES)
        qd = H.to_torch(q1, dtype, DEV)[None].contiguous()
        out = torch.empty((1, Hq, d), dtype=torch.float32, device=DEV)
        idx = torch.empty((1, Hq, k), dtype=torch.int32, device=DEV)
        vals = torch.empty((1, Hq, k), dtype=torch.float32, device=DEV)
        lse = torch.empty((1, Hq), dtype=torch.float32, device=DEV)
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            args = (cache.h, 0, qd.data_ptr(), k, W, out.data_ptr(), idx.data_ptr(), vals.data_ptr(), lse.data_ptr())
            ta.topk_attn_decode_window(*args, s.cuda_stream)   # warm-up outside the capture
            s.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                ta.topk_attn_decode_window(*args, s.cuda_stream)
            reads = []
            for rep, q in enumerate([q1, q2, q1, q2]):
                qd.copy_(H.to_torch(q, dtype, DEV)[None])      # eager work between replays
                out.zero_(); idx.zero_(); lse.zero_()
                s.synchronize()
                g.replay()
                s.synchronize()
                reads.append(ta.topk_attn_last_pages_read(cache.h)[0])
                H.check_unmargined((out[0].cpu().numpy(), idx[0].cpu().numpy(), vals[0].cpu().numpy(), lse[0].cpu().numpy()),
                                   q, K, V, dtype, k, W, f"pages replay {rep}")
                eager = cache.decode(0, qd, k, window=W)
                s.synchronize()
                assert torch.equal(eager[0], out) and torch.equal(eager[1], idx) and torch.equal(eager[3], lse)
            assert reads[0] == reads[2] and reads[1] == reads[3] and reads[0] != reads[1]
    finally:
        cache.close()


def test_c6_clustered_1m_tokens_sublinear_and_exact():
    """The clustered workload at full size (one million tokens, k = 16384, fp16): the page index reads a
    fraction of the pages and returns exactly the oracle's selection."""
    w = wl.C6
    q, K, V = wl.make_clustered(w, 0, 0.02, threads=16)
    q, K, V = wl.quantize(q, w.dtype), wl.quantize(K, w.dtype), wl.quantize(V, w.dtype)
    frac, _ = run_pages_case(q, K, V, w.dtype, w.k, label="c6")
    print(f"c6: {frac:.3f} of the pages read", flush=True)
    assert frac < 0.35


def test_pages_edge_cases_tiny_caches_reset_and_static_scratch():
    """Caches too short for the filtered scan, k beyond the cache, a sequence reset and filled again (its
    old balls must not survive), and the no-allocation entry point on a handle with a page index."""
    dtype, Hq, Hkv, d = wl.F16, 8, 2, 128
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, 70000, 900, dtype, index_kind=ta.INDEX_PAGES)
    try:
        cache.set_path(ta.PATH_PAGES)
        for N, k in ((100, 16), (70, 900), (3000, 64)):         # general path: every page read, result exact
            q, K, V = clustered(N, min(k, N), seed=N, sigma=0.05)
            cache.reset(0, 0)
            cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
            qd = H.to_torch(q, dtype, DEV)[None].contiguous()
            res = cache.decode(0, qd, k)
            torch.cuda.synchronize()
            read, total = ta.topk_attn_last_pages_read(cache.h)
            assert read == total == Hkv * ((N + PAGE - 1) // PAGE)
            H.check_unmargined(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, 0, f"pages tiny N={N} k={k}")
        # a long sequence after the short ones, appended in two pieces that split a page
        N, k = 69999, 700
        q, K, V = clustered(N, k, seed=5, sigma=0.02)
        cache.reset(0, 0)
        Kd, Vd = H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV)
        cache.append(0, 0, Kd[:, :33333].contiguous(), Vd[:, :33333].contiguous(), head_major=True)
        cache.append(0, 0, Kd[:, 33333:].contiguous(), Vd[:, 33333:].contiguous(), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        res = cache.decode(0, qd, k)
        torch.cuda.synchronize()
        read, total = ta.topk_attn_last_pages_read(cache.h)
        assert 0 < read < total
        H.check_unmargined(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, 0, "pages after reset")
        # the entry point that allocates nothing: same kernels on the library's own scratch array
        out = torch.empty_like(res[0]); idx = torch.empty_like(res[1]); vals = torch.empty_like(res[2]); lse = torch.empty_like(res[3])
        st = torch.cuda.current_stream(DEV).cuda_stream
        ta.topk_attn_decode_static(cache.h, 0, qd.data_ptr(), k, out.data_ptr(), idx.data_ptr(), vals.data_ptr(), lse.data_ptr(), st)
        torch.cuda.synchronize()
        assert torch.equal(out, res[0]) and torch.equal(idx, res[1]) and torch.equal(vals, res[2]) and torch.equal(lse, res[3])
    finally:
        cache.close()
