"""GPU tests of the compressed int8 key index (TOPK_ATTN_INDEX_INT8 / TOPK_ATTN_PATH_INDEX).

Bit-exact parts: the codes and scales the library keeps beside the keys, and the approximate
scores computed from them, against oracle/int8_index_ref.py.  The search itself is approximate
by contract: recall@k against the exact oracle (>= 0.999 per head; on inputs with a score
margin at the k-th boundary it is 1 in practice), every returned position carries its exact
score, and the attention output meets the usual tolerance.
"""
import ctypes

import numpy as np
import pytest
import torch

import helpers as H
from oracle import c_oracle
from oracle import int8_index_ref as i8
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl
from test_gpu_parity import rand_case

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None


def f32(x, dtype):
    return wl.widen(x, dtype).astype(np.float32)      # stored values are exactly representable


def index_views(cache, L, B, Hkv, Ncap, d):
    """Codes [L, B, Hkv, Ncap, d] int8 and scales [L, B, Hkv, Ncap] fp32 as laid out behind K and V."""
    up = lambda x: (x + 255) // 256 * 256
    rows = L * B * Hkv * Ncap
    half = up(rows * d * 2)
    codes = cache.kv[2 * half: 2 * half + rows * d].view(torch.int8).view(L, B, Hkv, Ncap, d)
    off = 2 * half + up(rows * d)
    scales = cache.kv[off: off + rows * 4].view(torch.float32).view(L, B, Hkv, Ncap)
    return codes, scales


@pytest.mark.parametrize("dtype,d", [(wl.F16, 128), (wl.BF16, 64), (wl.BF16, 128), (wl.F16, 256)])
def test_index_codes_and_scales_bit_exact(dtype, d):
    g = np.random.default_rng(d + dtype)
    L, B, Hq, Hkv, Ncap = 2, 2, 4, 2, 700
    K = g.standard_normal((Hkv, 650, d)).astype(np.float32) * g.uniform(0.01, 20.0, (Hkv, 650, 1)).astype(np.float32)
    K[0, 5] = 0.0                       # an all-zero row
    K[1, 9] = 1e-38                     # a row below the coding floor (bf16 keeps it, fp16 flushes it to 0)
    K[0, 11, 3] = 60000.0               # a huge outlier
    Ks = wl.quantize(K, dtype)
    Vs = wl.quantize(g.standard_normal((Hkv, 650, d)).astype(np.float32), dtype)
    cache = ta.TopkAttnCache(L, B, Hq, Hkv, d, Ncap, 16, dtype, index_kind=ta.INDEX_INT8)
    try:
        Kd, Vd = H.to_torch(Ks, dtype, DEV), H.to_torch(Vs, dtype, DEV)
        # layer 1, sequence 1, in three appends of uneven size (token-major for the middle one)
        cache.append(1, 1, Kd[:, :100].contiguous(), Vd[:, :100].contiguous(), head_major=True)
        cache.append(1, 1, Kd[:, 100:101].permute(1, 0, 2).contiguous(), Vd[:, 100:101].permute(1, 0, 2).contiguous())
        cache.append(1, 1, Kd[:, 101:].contiguous(), Vd[:, 101:].contiguous(), head_major=True)
        torch.cuda.synchronize()
        codes, scales = index_views(cache, L, B, Hkv, Ncap, d)
        want_c, want_s = i8.quantize_rows_int8(f32(Ks, dtype))
        np.testing.assert_array_equal(codes[1, 1, :, :650].cpu().numpy(), want_c)
        np.testing.assert_array_equal(scales[1, 1, :, :650].cpu().numpy(), want_s)
        assert (want_c[0, 5] == 0).all() and want_s[0, 5] == 0
    finally:
        cache.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,N,d", [(wl.F16, 8, 2, 3001, 128), (wl.BF16, 3, 3, 777, 64), (wl.F16, 4, 2, 64, 64),
                                                 (wl.BF16, 4, 1, 1000, 256)])
def test_index_approximate_scores_bit_exact(dtype, Hq, Hkv, N, d):
    q, K, V = rand_case(Hq, Hkv, N, d, dtype, N, seed=N)
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N + 50, 8, dtype, index_kind=ta.INDEX_INT8)
    try:
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        cache.set_path(ta.PATH_INDEX)
        got = cache.scores(0, H.to_torch(q, dtype, DEV)[None].contiguous())[0, :, :N].cpu().numpy()
        want = i8.approx_scores_int8(f32(q, dtype), f32(K, dtype))
        np.testing.assert_array_equal(got, want)
        cache.set_path(ta.PATH_AUTO)          # and the exact dump is still there
        exact = cache.scores(0, H.to_torch(q, dtype, DEV)[None].contiguous())[0, :, :N].cpu().numpy()
        ref = c_oracle.scores(q, K, dtype)
        assert np.abs(exact - ref).max() <= H.score_margin(q, K, dtype).max() / 8
    finally:
        cache.close()


def check_index_result(res, q, K, V, dtype, k, window=0, label="", margin_ok=True):
    """res: (out, idx, vals, lse) numpy [Hq, ...] from the index path; judged against the exact oracle.
    Without an enforced margin (`margin_ok` False) a head with full recall up to the rounding band is
    judged by helpers.check_unmargined."""
    out, idx, vals, lse = res
    Hq, d = q.shape
    N = K.shape[1]
    ref = c_oracle.topk_attention_window(q, K, V, dtype, k, window)
    delta = H.score_margin(q, K, dtype)
    k_eff = min(k, max(0, N - window))
    S = c_oracle.scores(q, K, dtype)
    recalls = [i8.recall_at_k(idx[h, :k_eff], ref[1][h, :k_eff]) for h in range(Hq)]
    assert min(recalls) >= 0.999, f"{label}: recall {min(recalls)}"
    for h in range(Hq if k_eff > 0 else 0):
        got = idx[h, :k_eff].astype(np.int64)
        assert len(set(got.tolist())) == k_eff and got.min() >= 0 and got.max() < N - window, f"{label}: bad positions"
        # every returned position carries its exact score
        assert np.abs(vals[h, :k_eff].astype(np.float64) - S[h, got]).max() <= delta[h] / 8, f"{label}: vals not exact"
    if not margin_ok:
        try:
            H.check_unmargined(res, q, K, V, dtype, k, window, label, S=S)
            return recalls
        except AssertionError as e:      # a key the index really missed (recall < 1): the looser bar below
            if "band" not in str(e):
                raise
    if min(recalls) == 1.0 and margin_ok:
        H.check_against_oracle(out, idx, vals, lse, ref, delta, k_eff, H.out_tolerance(dtype),
                               float(np.abs(wl.widen(V, dtype)).max()), label)
    else:   # a missed key sits at the k-th boundary and carries next to no softmax weight
        scale = np.maximum(np.abs(ref[0]).max(axis=1), 1e-6)
        assert (np.abs(out - ref[0]).max(axis=1) / scale).max() <= 5e-3, f"{label}: out"
    return recalls


def run_index_case(q, K, V, dtype, k, window=0, label="", expect_fallbacks=0, margin_ok=True):
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    cache = ta.TopkAttnCache(1, 1, Hq, Hkv, d, N, k, dtype, max_window=window, index_kind=ta.INDEX_INT8)
    try:
        cache.set_path(ta.PATH_INDEX)
        cache.append(0, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = H.to_torch(q, dtype, DEV)[None].contiguous()
        res = cache.decode(0, qd, k, window=window)
        torch.cuda.synchronize()
        fb = cache.last_fallbacks()
        rec = check_index_result(tuple(t[0].cpu().numpy() for t in res), q, K, V, dtype, k, window, label, margin_ok)
        if expect_fallbacks is not None:
            assert fb == expect_fallbacks, f"{label}: {fb} heads fell back"
        res2 = cache.decode(0, qd, k, window=window)          # repeatable
        torch.cuda.synchronize()
        for a, b in zip(res, res2):
            assert torch.equal(a, b)
        return rec
    finally:
        cache.close()


@pytest.mark.parametrize("dtype,Hq,Hkv,N,d,k,window", [
    (wl.F16, 8, 2, 40000, 128, 300, 0),
    (wl.BF16, 8, 2, 65536 + 17, 128, 1024, 0),
    (wl.F16, 4, 2, 50000, 64, 64, 0),          # G = 2, d = 64
    (wl.BF16, 3, 3, 33333, 128, 500, 0),       # G = 1
    (wl.F16, 12, 4, 70001, 128, 1, 0),         # G = 3, k = 1
    (wl.F16, 8, 2, 40000, 128, 400, 1000),     # with the recent-token window
    (wl.BF16, 4, 2, 45000, 256, 500, 0),       # d = 256
])
def test_index_decode_recall(dtype, Hq, Hkv, N, d, k, window):
    g = np.random.default_rng(N + k)
    q = wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), dtype)
    K = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    V = wl.quantize(g.standard_normal((Hkv, N, d)).astype(np.float32), dtype)
    P = N - window
    Kp = np.ascontiguousarray(K[:, :P])
    Kp, _, _ = H.enforce_margin(q, Kp, dtype, k)
    K[:, :P] = Kp
    run_index_case(q, K, V, dtype, k, window, label=f"index N={N} k={k} W={window}")


def test_index_recall_on_raw_workload_without_margin():
    """The 128k-token bf16 configuration as generated (no score margin enforced, outlier
    channels in K): recall and output tolerance only."""
    w = wl.C2
    q, K, V = wl.make_quantized(w, 1)
    cache = ta.TopkAttnCache(1, 1, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_tokens, w.k, w.dtype,
                             index_kind=ta.INDEX_INT8)
    try:
        cache.set_path(ta.PATH_INDEX)
        cache.append(0, 0, H.to_torch(K, w.dtype, DEV), H.to_torch(V, w.dtype, DEV), head_major=True)
        out, idx, vals, lse = cache.decode(0, H.to_torch(q, w.dtype, DEV)[None].contiguous(), w.k)
        torch.cuda.synchronize()
        assert cache.last_fallbacks() == 0
        ref = c_oracle.topk_attention(q, K, V, w.dtype, w.k)
        rec = [i8.recall_at_k(idx[0, h].cpu().numpy(), ref[1][h]) for h in range(w.n_q_heads)]
        assert min(rec) >= 0.999, rec
        o = out[0].cpu().numpy()
        scale = np.maximum(np.abs(ref[0]).max(axis=1), 1e-6)
        assert (np.abs(o - ref[0]).max(axis=1) / scale).max() <= 2e-3
    finally:
        cache.close()


def test_index_short_cache_and_dense_k_use_the_exact_path():
    """Where the filtered scan does not apply the index path is the exact path."""
    for N, k in [(500, 20), (20000, 9000)]:
        q, K, V = rand_case(8, 2, N, 128, wl.F16, k, seed=N)
        rec = run_index_case(q, K, V, wl.F16, k, label=f"index->exact N={N} k={k}")
        assert min(rec) == 1.0


def test_index_ragged_batch_path_switch_and_errors():
    dtype, Hq, Hkv, d, k = wl.BF16, 8, 2, 128, 150
    lens = [40000, 34001, 33000]
    cache = ta.TopkAttnCache(1, 3, Hq, Hkv, d, max(lens), k, dtype, index_kind=ta.INDEX_INT8, max_queries=2)
    plain = ta.TopkAttnCache(1, 1, Hq, Hkv, d, 64, 8, dtype)
    try:
        assert ta.lib().topk_attn_set_path(plain.h, ta.PATH_INDEX) == ta.EINVAL      # no index configured
        assert ta.lib().topk_attn_set_path(cache.h, 4) == ta.EINVAL
        data = []
        for b, n in enumerate(lens):
            q, K, V = rand_case(Hq, Hkv, n, d, dtype, k, seed=500 + b)
            data.append((q, K, V))
            cache.append(0, b, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
        qd = torch.stack([H.to_torch(x[0], dtype, DEV) for x in data]).contiguous()
        exact = cache.decode(0, qd, k)                         # default path: exact
        cache.set_path(ta.PATH_INDEX)
        approx = cache.decode(0, qd, k)
        torch.cuda.synchronize()
        assert cache.last_fallbacks() == 0
        for b in range(3):
            q, K, V = data[b]
            check_index_result(tuple(t[b].cpu().numpy() for t in approx), q, K, V, dtype, k, 0, f"ragged index seq {b}")
        assert torch.equal(torch.sort(exact[1], dim=-1).values, torch.sort(approx[1], dim=-1).values)
        # several queries per sequence are served by the exact path also under PATH_INDEX
        q2 = torch.stack([qd, qd], dim=1).contiguous()         # [B, 2, Hq, d]
        multi = cache.decode_multi(0, q2, k, causal=False)
        torch.cuda.synchronize()
        assert torch.equal(torch.sort(multi[1][:, 1], dim=-1).values, torch.sort(exact[1], dim=-1).values)
    finally:
        cache.close()
        plain.close()


def test_c3_index_decode_1m_fp16():
    """The N = 1M configuration through the int8 index."""
    w = wl.C3
    q, K, V = wl.make_quantized(w, 0, threads=16)
    K, _, _ = H.enforce_margin(q, K, w.dtype, w.k)
    rec = run_index_case(q, K, V, w.dtype, w.k, label="c3 index")
    assert min(rec) == 1.0


def test_index_layer_schedule_in_one_call():
    """Three layers with their own k through topk_attn_decode_layers under the index path:
    each layer judged against the exact oracle, and bit-identical to separate calls."""
    dtype, L, Hq, Hkv, d, N = wl.F16, 3, 8, 2, 128, 36000
    ks = ta.topk_attn_k_schedule(900, L, 2.0)
    cache = ta.TopkAttnCache(L, 1, Hq, Hkv, d, N, max(ks), dtype, index_kind=ta.INDEX_INT8)
    try:
        cache.set_path(ta.PATH_INDEX)
        data, queries, single = [], [], []
        for l in range(L):
            q, K, V = rand_case(Hq, Hkv, N, d, dtype, ks[l], seed=600 + l)
            data.append((q, K, V))
            cache.append(l, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
            queries.append(H.to_torch(q, dtype, DEV)[None].contiguous())
            single.append(cache.decode(l, queries[-1], ks[l]))
        qd = torch.stack(queries).contiguous()
        out = torch.empty((L, 1, Hq, d), dtype=torch.float32, device=DEV)
        idx = torch.empty((Hq * sum(ks),), dtype=torch.int32, device=DEV)
        vals = torch.empty((Hq * sum(ks),), dtype=torch.float32, device=DEV)
        lse = torch.empty((L, 1, Hq), dtype=torch.float32, device=DEV)
        ta.topk_attn_decode_layers(cache.h, 0, ks, qd.data_ptr(), 0, out.data_ptr(), idx.data_ptr(), vals.data_ptr(),
                                   lse.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        off = 0
        for l in range(L):
            n = Hq * ks[l]
            q, K, V = data[l]
            res = (out[l, 0].cpu().numpy(), idx[off:off + n].view(Hq, ks[l]).cpu().numpy(),
                   vals[off:off + n].view(Hq, ks[l]).cpu().numpy(), lse[l, 0].cpu().numpy())
            check_index_result(res, q, K, V, dtype, ks[l], 0, f"index layer {l} k={ks[l]}")
            assert torch.equal(out[l], single[l][0]) and torch.equal(idx[off:off + n].view(1, Hq, ks[l]), single[l][1])
            off += n
    finally:
        cache.close()


def test_c4_batched_index_decode():
    """Config 4 at full size (16 sequences x 262144 tokens, bf16) through the int8 index, k = 1024;
    two sequences are checked against the exact oracle, all of them for self-consistency
    with the exact path of the library."""
    w = wl.C4
    B, Hq, Hkv, d, N, k = w.n_seqs, w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_tokens, 1024
    sampled = [0, 15]
    cache = ta.TopkAttnCache(1, B, Hq, Hkv, d, N, k, w.dtype, index_kind=ta.INDEX_INT8)
    try:
        host, qs = {}, []
        for b in range(B):
            q, K, V = wl.make_quantized(w, seed=3, seq=b, threads=16)
            if b in sampled:
                K, _, _ = H.enforce_margin(q, K, w.dtype, k)
                host[b] = (q, K, V)
            cache.append(0, b, H.to_torch(K, w.dtype, DEV), H.to_torch(V, w.dtype, DEV), head_major=True)
            qs.append(H.to_torch(q, w.dtype, DEV))
        qd = torch.stack(qs).contiguous()
        exact = cache.decode(0, qd, k)
        cache.set_path(ta.PATH_INDEX)
        approx = cache.decode(0, qd, k)
        torch.cuda.synchronize()
        assert cache.last_fallbacks() == 0
        for b in sampled:
            q, K, V = host[b]
            check_index_result(tuple(t[b].cpu().numpy() for t in approx), q, K, V, w.dtype, k, 0, f"c4 index seq {b}")
        # every sequence: at least 99.9 % of the exact path's positions, per head
        se, sa = torch.sort(exact[1], dim=-1).values, torch.sort(approx[1], dim=-1).values
        same = (se == sa).all(dim=-1)
        for b, h in (~same).nonzero().tolist():
            rec = i8.recall_at_k(approx[1][b, h].cpu().numpy(), exact[1][b, h].cpu().numpy())
            assert rec >= 0.999, (b, h, rec)
        np.testing.assert_allclose(approx[0].cpu().numpy(), exact[0].cpu().numpy(), rtol=0, atol=5e-3 * float(exact[0].abs().max()))
    finally:
        cache.close()
