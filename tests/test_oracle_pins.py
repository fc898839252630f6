"""Pins for the CPU oracles (NumPy and plain C).  CPU only.

Each test ties the oracle to something that is not the oracle: a library
routine (dense attention, sort, argpartition), a closed form, brute force on
tiny inputs or an invariant of the definition.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import c_oracle
from oracle import topk_attention_ref as ref
from paper_2502_06766_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(Hq, Hkv, N, d, seed, dtype=wl.F32):
    g = np.random.default_rng(seed)
    q = g.standard_normal((Hq, d)).astype(np.float32)
    K = g.standard_normal((Hkv, N, d)).astype(np.float32)
    V = g.standard_normal((Hkv, N, d)).astype(np.float32)
    qs, Ks, Vs = wl.quantize(q, dtype), wl.quantize(K, dtype), wl.quantize(V, dtype)
    return (qs, Ks, Vs), (wl.widen(qs, dtype), wl.widen(Ks, dtype), wl.widen(Vs, dtype))


def _dense_library(q, K, V):
    """Eq. 1 through torch's scaled_dot_product_attention (float64, CPU), with the
    library's own GQA convention (query head h -> KV head h // G)."""
    Hq, d = q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    qt = torch.from_numpy(q)[None, :, None, :]
    Kt = torch.from_numpy(K).repeat_interleave(G, dim=0)[None]
    Vt = torch.from_numpy(V).repeat_interleave(G, dim=0)[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)
    return o[0, :, 0, :].numpy()


# ---------------------------------------------------------------- k = N is Eq. 1
@pytest.mark.parametrize("Hq,Hkv,N,d", [(1, 1, 37, 8), (4, 2, 129, 16), (8, 2, 300, 64)])
def test_k_equals_n_is_dense_attention_numpy(Hq, Hkv, N, d):
    _, (q, K, V) = _rand(Hq, Hkv, N, d, 1)
    out, idx, vals, lse = ref.topk_attention(q, K, V, N)
    np.testing.assert_allclose(out, _dense_library(q, K, V), rtol=1e-12, atol=1e-13)
    for h in range(Hq):
        assert sorted(idx[h].tolist()) == list(range(N))
    # lse against the library's logsumexp
    G = Hq // Hkv
    for h in range(Hq):
        z = torch.from_numpy(K[h // G] @ q[h]) / math.sqrt(d)
        assert abs(lse[h] - float(torch.logsumexp(z, 0))) < 1e-12


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_k_equals_n_is_dense_attention_c(dtype):
    (qs, Ks, Vs), (q, K, V) = _rand(8, 2, 257, 32, 2, dtype)
    out, idx, vals, lse = c_oracle.topk_attention(qs, Ks, Vs, dtype, 257)
    np.testing.assert_allclose(out, _dense_library(q, K, V), rtol=1e-12, atol=1e-13)
    # k > N pads and changes nothing else
    out2, idx2, vals2, _ = c_oracle.topk_attention(qs, Ks, Vs, dtype, 300)
    np.testing.assert_allclose(out2, out, rtol=0, atol=0)
    assert (idx2[:, 257:] == -1).all() and np.isneginf(vals2[:, 257:]).all()
    assert (idx2[:, :257] == idx).all()


# ---------------------------------------------------------------- closed form
def test_closed_form_log_scores():
    """d = 4 so sqrt(d) = 2; q = (2,0,0,0) and key i = (ln(i+1),0,0,0) give scaled
    scores ln(i+1), i.e. softmax weights proportional to i+1.  With N = 5, k = 3
    the selected positions are {4,3,2} with weights 5/12, 4/12, 3/12 and
    lse = ln 12; vals are the raw scores 2 ln(i+1)."""
    N, d, k = 5, 4, 3
    q = np.array([[2.0, 0, 0, 0]])
    K = np.zeros((1, N, d))
    K[0, :, 0] = np.log(np.arange(1, N + 1))
    V = np.arange(N * d, dtype=np.float64).reshape(1, N, d) ** 1.5
    want = (5 * V[0, 4] + 4 * V[0, 3] + 3 * V[0, 2]) / 12.0
    out, idx, vals, lse = ref.topk_attention(q, K, V, k)
    np.testing.assert_allclose(out[0], want, rtol=1e-13)
    assert idx[0].tolist() == [4, 3, 2]
    np.testing.assert_allclose(vals[0], 2 * np.log([5, 4, 3]), rtol=1e-14)
    assert abs(lse[0] - math.log(12.0)) < 1e-13
    # same case through the C oracle (fp32 storage: compare against the rounded inputs)
    qs, Ks, Vs = (a.astype(np.float32) for a in (q, K, V))
    out_c, idx_c, vals_c, lse_c = c_oracle.topk_attention(qs, Ks, Vs, wl.F32, k)
    w = np.exp(Ks[0, [4, 3, 2], 0].astype(np.float64))   # exp(ln(i+1)) up to fp32 rounding
    want_c = (w[:, None] * Vs[0, [4, 3, 2]].astype(np.float64)).sum(0) / w.sum()
    np.testing.assert_allclose(out_c[0], want_c, rtol=1e-13)
    assert idx_c[0].tolist() == [4, 3, 2]
    assert abs(lse_c[0] - math.log(12.0)) < 1e-6


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(6))
def test_bruteforce_subsets_tiny(seed):
    """For tie-free scores the top-k set is the unique k-subset with the largest
    score sum; the output is the explicit softmax-weighted sum over it."""
    g = np.random.default_rng(seed)
    N, d, k = int(g.integers(5, 12)), 4, int(g.integers(1, 5))
    (qs, Ks, Vs), (q, K, V) = _rand(2, 1, N, d, 100 + seed)
    S = [[sum(q[h, c] * K[0, i, c] for c in range(d)) for i in range(N)] for h in range(2)]
    out, idx, vals, lse = ref.topk_attention(q, K, V, k)
    out_c, idx_c, vals_c, _ = c_oracle.topk_attention(qs, Ks, Vs, wl.F32, k)
    for h in range(2):
        best = max(itertools.combinations(range(N), k), key=lambda I: sum(S[h][i] for i in I))
        assert set(idx[h].tolist()) == set(best)
        assert set(idx_c[h].tolist()) == set(best)
        mx = max(S[h][i] for i in best)
        w = {i: math.exp((S[h][i] - mx) / math.sqrt(d)) for i in best}
        Z = sum(w.values())
        want = [sum(w[i] / Z * V[0, i, c] for i in best) for c in range(d)]
        np.testing.assert_allclose(out[h], want, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(out_c[h], want, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(sorted(vals[h]), sorted(S[h][i] for i in best), rtol=1e-13)


# ---------------------------------------------------------------- library selection
@pytest.mark.parametrize("N,k", [(1000, 1), (1000, 17), (5000, 500), (4096, 4096)])
def test_selection_matches_library_partition(N, k):
    (qs, Ks, Vs), (q, K, V) = _rand(4, 2, N, 16, 7)
    S = ref.scores(q, K)
    _, idx, vals, _ = ref.topk_attention(q, K, V, k)
    _, idx_c, vals_c, _ = c_oracle.topk_attention(qs, Ks, Vs, wl.F32, k)
    for h in range(4):
        part = np.argpartition(-S[h], k - 1)[:k] if k < N else np.arange(N)
        assert set(idx[h].tolist()) == set(part.tolist())
        assert set(idx_c[h].tolist()) == set(part.tolist())
        np.testing.assert_array_equal(vals[h], np.sort(S[h])[::-1][:k])
        np.testing.assert_allclose(vals_c[h], vals[h], rtol=1e-13, atol=1e-13)
        rest = np.setdiff1d(np.arange(N), idx[h])
        if rest.size:
            assert vals[h].min() >= S[h][rest].max()
        # vals are the raw dot products of the selected keys (unscaled)
        np.testing.assert_allclose(vals[h], K[h // 2][idx[h]] @ q[h], rtol=1e-13)


def test_scores_orientation_and_gqa_mapping():
    """scores[h, i] = q_h . K[h // G, i]: check against an explicit einsum per KV
    head with distinct caches per head (catches transposed or mis-grouped heads)."""
    (qs, Ks, _), (q, K, _) = _rand(6, 3, 50, 8, 3)
    want = np.einsum("hgd,hnd->hgn", q.reshape(3, 2, 8), K).reshape(6, 50)
    np.testing.assert_allclose(ref.scores(q, K), want, rtol=1e-13)
    np.testing.assert_allclose(c_oracle.scores(qs, Ks, wl.F32), want, rtol=1e-13)


# ---------------------------------------------------------------- special cases
def test_k1_returns_argmax_value_row():
    (qs, Ks, Vs), (q, K, V) = _rand(4, 2, 333, 16, 11)
    out, idx, _, lse = ref.topk_attention(q, K, V, 1)
    out_c, idx_c, _, _ = c_oracle.topk_attention(qs, Ks, Vs, wl.F32, 1)
    for h in range(4):
        i = int(np.argmax(K[h // 2] @ q[h]))
        assert idx[h, 0] == i and idx_c[h, 0] == i
        np.testing.assert_array_equal(out[h], V[h // 2, i])
        np.testing.assert_array_equal(out_c[h], V[h // 2, i])
        assert abs(lse[h] - (K[h // 2, i] @ q[h]) / 4.0) < 1e-13


def test_identical_keys_tie_rule_and_mean():
    """All scores equal: lowest positions win and the output is their mean."""
    N, d, k = 40, 8, 7
    g = np.random.default_rng(5)
    q = g.standard_normal((1, d))
    K = np.tile(g.standard_normal((1, 1, d)), (1, N, 1))
    V = g.standard_normal((1, N, d))
    out, idx, _, _ = ref.topk_attention(q, K, V, k)
    assert idx[0].tolist() == list(range(k))
    np.testing.assert_allclose(out[0], V[0, :k].mean(0), rtol=1e-13)
    f = lambda a: a.astype(np.float32)
    out_c, idx_c, _, _ = c_oracle.topk_attention(f(q), f(K), f(V), wl.F32, k)
    assert idx_c[0].tolist() == list(range(k))
    np.testing.assert_allclose(out_c[0], f(V)[0, :k].astype(np.float64).mean(0), rtol=1e-13)


def test_duplicate_key_pairs_tie_rule():
    """Key j+N/2 duplicates key j: when only one of a pair fits, the lower position wins."""
    (_, _, _), (q, K, V) = _rand(1, 1, 64, 8, 21)
    K[0, 32:] = K[0, :32]
    for k in (1, 3, 9):
        _, idx, _, _ = ref.topk_attention(q, K, V, k)
        order = np.argsort(-(K[0, :32] @ q[0]), kind="stable")
        want = []
        for j in order:
            want += [int(j), int(j) + 32]
        assert idx[0].tolist() == want[:k]


def test_score_shift_and_query_scale_invariance():
    (_, _, _), (q, K, V) = _rand(2, 1, 400, 16, 31)
    out, idx, vals, _ = ref.topk_attention(q[:1], K, V, 25)
    # adding c q/|q|^2 to every key shifts every score by c: same set, same output
    c = 3.25
    K2 = K + c * q[0] / (q[0] @ q[0])
    out2, idx2, vals2, _ = ref.topk_attention(q[:1], K2, V, 25)
    assert idx2[0].tolist() == idx[0].tolist()
    np.testing.assert_allclose(vals2[0], vals[0] + c, rtol=1e-12)
    np.testing.assert_allclose(out2, out, rtol=1e-10)
    # scaling the query by a > 0 keeps the selected set (the metric is the raw dot product)
    _, idx3, vals3, _ = ref.topk_attention(2.5 * q[:1], K, V, 25)
    assert idx3[0].tolist() == idx[0].tolist()
    np.testing.assert_allclose(vals3[0], 2.5 * vals[0], rtol=1e-13)


def test_permutation_invariance():
    (_, _, _), (q, K, V) = _rand(4, 2, 500, 16, 41)
    out, idx, _, _ = ref.topk_attention(q, K, V, 33)
    perm = np.random.default_rng(0).permutation(500)     # new position j holds old row perm[j]
    out_p, idx_p, _, _ = ref.topk_attention(q, K[:, perm], V[:, perm], 33)
    np.testing.assert_allclose(out_p, out, rtol=1e-11, atol=1e-13)
    for h in range(4):
        assert set(perm[idx_p[h]].tolist()) == set(idx[h].tolist())


def test_planted_dominant_keys_are_selected():
    w = wl.C1
    q, K, V = wl.make_cache(w, seed=0)
    q, K, V = q.astype(np.float64), K.astype(np.float64), V.astype(np.float64)
    S = ref.scores(q, K)[0]
    g = np.random.default_rng(9)
    planted = g.choice(w.n_tokens, size=5, replace=False)
    # rescale each planted row so its score is 1.5x the largest other score
    top_other = np.delete(S, planted).max()
    for p in planted:
        K[0, p] = q[0] * (1.5 * top_other / (q[0] @ q[0]))
    _, idx, _, _ = ref.topk_attention(q, K, V, 5)
    assert set(idx[0].tolist()) == set(planted.tolist())
    _, idx, _, _ = ref.topk_attention(q, K, V, 64)
    assert set(planted.tolist()) <= set(idx[0].tolist())


def test_weights_sum_to_one_and_convex_hull():
    (_, _, _), (q, K, V) = _rand(2, 2, 300, 8, 51)
    out, idx, vals, lse = ref.topk_attention(q, K, V, 20)
    for h in range(2):
        rows = V[h][idx[h]]
        assert (out[h] <= rows.max(0) + 1e-12).all() and (out[h] >= rows.min(0) - 1e-12).all()
        p = np.exp(vals[h] / math.sqrt(8) - lse[h])
        assert abs(p.sum() - 1.0) < 1e-12
        np.testing.assert_allclose(out[h], p @ rows, rtol=1e-12)


def test_truncation_error_bound():
    """|out_topk - out_dense|_inf <= 2 (1 - m) max|V| with m the dense mass captured."""
    w = wl.C5.scaled(8192, k=164, n_layers=1)
    qs, Ks, Vs = wl.make_quantized(w, seed=3)
    q, K, V = (wl.widen(a, w.dtype) for a in (qs, Ks, Vs))
    out, idx, _, _ = ref.topk_attention(q, K, V, w.k)
    dense = _dense_library(q, K, V)
    S = ref.scores(q, K)
    masses = []
    for h in range(w.n_q_heads):
        m = ref.captured_mass(S[h], idx[h], w.head_dim)
        masses.append(m)
        bound = 2 * (1 - m) * np.abs(V[h // w.group]).max()
        assert np.abs(out[h] - dense[h]).max() <= bound + 1e-12
    # the score-shaped recipe concentrates ~95 % of the dense mass on the top 2 %
    assert 0.85 < float(np.mean(masses)) < 0.99
    ent = np.mean([ref.attention_entropy(S[h], w.head_dim) for h in range(w.n_q_heads)])
    assert ent < math.log(w.n_tokens)


def test_entropy_uniform_is_log_n():
    assert abs(ref.attention_entropy(np.full(1000, 0.37), 64) - math.log(1000)) < 1e-12
    assert ref.attention_entropy(np.array([0.0, 1000.0, 0.0]), 1) < 1e-12


# ---------------------------------------------------------------- C vs NumPy, dtypes
@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("Hq,Hkv,N,d,k", [(4, 1, 700, 64, 50), (8, 2, 1025, 128, 128), (2, 2, 64, 8, 64)])
def test_c_oracle_matches_numpy_oracle(dtype, Hq, Hkv, N, d, k):
    (qs, Ks, Vs), (q, K, V) = _rand(Hq, Hkv, N, d, 61, dtype)
    out, idx, vals, lse = ref.topk_attention(q, K, V, k)
    out_c, idx_c, vals_c, lse_c = c_oracle.topk_attention(qs, Ks, Vs, dtype, k)
    np.testing.assert_array_equal(idx_c, idx)
    np.testing.assert_allclose(vals_c, vals, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(out_c, out, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse_c, lse, rtol=1e-13)
    np.testing.assert_allclose(c_oracle.scores(qs, Ks, dtype), ref.scores(q, K), rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
def test_c_oracle_widens_every_16bit_pattern_exactly(dtype):
    """q = [1], one key per finite 16-bit pattern: scores must be the stored values."""
    bits = np.arange(65536, dtype=np.uint16)
    if dtype == wl.F16:
        vals = bits.view(np.float16).astype(np.float64)
        K = bits.view(np.float16)[None, :, None]
        q = np.array([[1.0]], dtype=np.float16)
    else:
        vals = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
        K = bits[None, :, None]
        q = wl.to_bf16_bits(np.array([[1.0]], dtype=np.float32))
    S = c_oracle.scores(q, np.ascontiguousarray(K), dtype)[0]
    fin = np.isfinite(vals)
    np.testing.assert_array_equal(S[fin], vals[fin])


def test_bf16_rounding_matches_library():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(wl.to_bf16_bits(x), lib)
    np.testing.assert_array_equal(wl.bf16_bits_to_f32(lib),
                                  torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())


# ---------------------------------------------------------------- sizes the paper prints
def test_kv_cache_sizes_printed_in_paper():
    for line in open(os.path.join(GOLDEN, "kv_cache_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, hidden, layers, bpe, gb = line.split()
        got = wl.kv_cache_bytes(int(n), int(hidden), int(layers), int(bpe)) / 1e9
        assert abs(got - float(gb)) / float(gb) < 0.03, (line, got)


# ---------------------------------------------------------------- recent-token window (Algorithm 1's K_gen / V_gen)
def test_window_zero_is_plain_topk():
    (qs, Ks, Vs), (q, K, V) = _rand(4, 2, 200, 16, 71)
    a = ref.topk_attention(q, K, V, 17)
    b = ref.topk_attention_window(q, K, V, 17, 0)
    c = c_oracle.topk_attention_window(qs, Ks, Vs, wl.F32, 17, 0)
    for x, y, z in zip(a, b, c):
        np.testing.assert_array_equal(x, y)
        np.testing.assert_allclose(z, x, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("N,k,W", [(60, 50, 10), (60, 100, 7), (33, 5, 33), (33, 5, 80)])
def test_window_covering_everything_is_dense_attention(N, k, W):
    """k >= N - W (or W >= N): every cached token is attended, so the result is Eq. 1."""
    (qs, Ks, Vs), (q, K, V) = _rand(4, 2, N, 8, 72)
    dense = _dense_library(q, K, V)
    out, idx, vals, lse = ref.topk_attention_window(q, K, V, k, W)
    out_c, idx_c, _, lse_c = c_oracle.topk_attention_window(qs, Ks, Vs, wl.F32, k, W)
    np.testing.assert_allclose(out, dense, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(out_c, dense, rtol=1e-12, atol=1e-13)
    P = max(0, N - W)
    for h in range(4):
        assert sorted(i for i in idx[h].tolist() if i >= 0) == list(range(min(k, P)))
        assert (idx[h][min(k, P):] == -1).all()
        z = torch.from_numpy(K[h // 2] @ q[h]) / math.sqrt(8)
        assert abs(lse[h] - float(torch.logsumexp(z, 0))) < 1e-12
        assert abs(lse_c[h] - lse[h]) < 1e-12
    np.testing.assert_array_equal(idx_c, idx)


@pytest.mark.parametrize("seed", range(4))
def test_window_bruteforce_tiny(seed):
    g = np.random.default_rng(seed)
    N, d = int(g.integers(8, 13)), 4
    W, k = int(g.integers(1, 4)), int(g.integers(1, 4))
    (qs, Ks, Vs), (q, K, V) = _rand(1, 1, N, d, 200 + seed)
    P = N - W
    S = [sum(q[0, c] * K[0, i, c] for c in range(d)) for i in range(N)]
    best = max(itertools.combinations(range(P), k), key=lambda I: sum(S[i] for i in I))
    att = list(best) + list(range(P, N))
    mx = max(S[i] for i in att)
    w = {i: math.exp((S[i] - mx) / math.sqrt(d)) for i in att}
    Z = sum(w.values())
    want = [sum(w[i] / Z * V[0, i, c] for i in att) for c in range(d)]
    for out, idx, vals, lse in (ref.topk_attention_window(q, K, V, k, W),
                                c_oracle.topk_attention_window(qs, Ks, Vs, wl.F32, k, W)):
        assert set(idx[0].tolist()) == set(best)
        np.testing.assert_allclose(out[0], want, rtol=1e-12, atol=1e-14)
        assert abs(lse[0] - (mx / math.sqrt(d) + math.log(Z))) < 1e-12


def test_window_is_lse_merge_of_topk_prefix_and_dense_window():
    """out = (e^la out_a + e^lb out_b) / (e^la + e^lb) with a = top-k attention over the
    prefix alone and b = dense attention (library) over the window alone."""
    (qs, Ks, Vs), (q, K, V) = _rand(6, 3, 500, 16, 73)
    k, W = 40, 37
    P = 500 - W
    out_a, idx_a, vals_a, lse_a = ref.topk_attention(q, K[:, :P], V[:, :P], k)
    out_b = _dense_library(q, K[:, P:], V[:, P:])
    out, idx, vals, lse = ref.topk_attention_window(q, K, V, k, W)
    out_c, idx_c, vals_c, lse_c = c_oracle.topk_attention_window(qs, Ks, Vs, wl.F32, k, W)
    np.testing.assert_array_equal(idx, idx_a)
    np.testing.assert_array_equal(idx_c, idx_a)
    for h in range(6):
        lb = float(torch.logsumexp(torch.from_numpy(K[h // 2, P:] @ q[h]) / 4.0, 0))
        wa, wb = math.exp(lse_a[h] - lse[h]), math.exp(lb - lse[h])
        assert abs(wa + wb - 1.0) < 1e-12
        np.testing.assert_allclose(out[h], wa * out_a[h] + wb * out_b[h], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(out_c[h], out[h], rtol=1e-11, atol=1e-13)
        assert abs(lse_c[h] - lse[h]) < 1e-12


# ---------------------------------------------------------------- several queries per cache
def _rand_multi(M, Hq, Hkv, N, d, seed, dtype=wl.F32):
    g = np.random.default_rng(seed)
    q = g.standard_normal((M, Hq, d)).astype(np.float32)
    K = g.standard_normal((Hkv, N, d)).astype(np.float32)
    V = g.standard_normal((Hkv, N, d)).astype(np.float32)
    qs, Ks, Vs = wl.quantize(q, dtype), wl.quantize(K, dtype), wl.quantize(V, dtype)
    return (qs, Ks, Vs), (wl.widen(qs, dtype), wl.widen(Ks, dtype), wl.widen(Vs, dtype))


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16])
def test_multi_causal_with_k_at_least_n_is_library_causal_attention(dtype):
    """With k >= N every visible key is selected, so a causal chunk of M queries is the
    last M rows of causal dense attention (library routine with a boolean mask)."""
    M, Hq, Hkv, N, d = 5, 4, 2, 70, 16
    (qs, Ks, Vs), (q, K, V) = _rand_multi(M, Hq, Hkv, N, d, 310, dtype)
    G = Hq // Hkv
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]                         # [1, Hq, M, d]
    Kt = torch.from_numpy(K).repeat_interleave(G, dim=0)[None]
    Vt = torch.from_numpy(V).repeat_interleave(G, dim=0)[None]
    pos = torch.arange(N)[None, :]
    mask = pos <= (N - M + torch.arange(M))[:, None]                        # query m sees tokens 0 .. N-M+m
    want = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    for out, idx, vals, lse in (ref.topk_attention_multi(q, K, V, N, True),
                                c_oracle.topk_attention_multi(qs, Ks, Vs, dtype, N, True)):
        np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-13)
        for m in range(M):
            n_vis = N - (M - 1 - m)
            for h in range(Hq):
                assert sorted(i for i in idx[m, h].tolist() if i >= 0) == list(range(n_vis))
                assert (idx[m, h] == -1).sum() == N - n_vis


def test_multi_rows_are_single_query_steps():
    """Non-causal: row m is the plain step for query m.  Causal: the last query sees the
    whole cache (plain step), the first one a cache M - 1 tokens shorter."""
    M, Hq, Hkv, N, d, k = 3, 6, 2, 200, 8, 17
    (qs, Ks, Vs), (q, K, V) = _rand_multi(M, Hq, Hkv, N, d, 311)
    for fn_multi, fn_one, args in ((lambda c: ref.topk_attention_multi(q, K, V, k, c),
                                    lambda m, n: ref.topk_attention(q[m], K[:, :n], V[:, :n], k), None),
                                   (lambda c: c_oracle.topk_attention_multi(qs, Ks, Vs, wl.F32, k, c),
                                    lambda m, n: c_oracle.topk_attention(
                                        qs[m], np.ascontiguousarray(Ks[:, :n]), np.ascontiguousarray(Vs[:, :n]),
                                        wl.F32, k), None)):
        out, idx, vals, lse = fn_multi(False)
        for m in range(M):
            o1, i1, v1, l1 = fn_one(m, N)
            np.testing.assert_array_equal(idx[m], i1)
            np.testing.assert_allclose(out[m], o1, rtol=1e-13, atol=0)
        out, idx, vals, lse = fn_multi(True)
        for m in (0, M - 1):
            o1, i1, v1, l1 = fn_one(m, N - (M - 1 - m))
            np.testing.assert_array_equal(idx[m], i1)
            np.testing.assert_allclose(out[m], o1, rtol=1e-13, atol=0)
            np.testing.assert_allclose(lse[m], l1, rtol=1e-13, atol=0)
        assert idx[0].max() <= N - M        # the first query never sees the last M - 1 tokens


@pytest.mark.parametrize("seed", range(3))
def test_multi_bruteforce_tiny(seed):
    g = np.random.default_rng(900 + seed)
    N, d, M = int(g.integers(9, 13)), 4, 3
    k, W = int(g.integers(1, 4)), int(g.integers(0, 3))
    (qs, Ks, Vs), (q, K, V) = _rand_multi(M, 1, 1, N, d, 320 + seed)
    res = (ref.topk_attention_multi(q, K, V, k, True, W), c_oracle.topk_attention_multi(qs, Ks, Vs, wl.F32, k, True, W))
    for m in range(M):
        n_vis = N - (M - 1 - m)
        P = n_vis - W
        S = [sum(q[m, 0, c] * K[0, i, c] for c in range(d)) for i in range(n_vis)]
        best = max(itertools.combinations(range(P), k), key=lambda I: sum(S[i] for i in I))
        att = list(best) + list(range(P, n_vis))
        mx = max(S[i] for i in att)
        w = {i: math.exp((S[i] - mx) / math.sqrt(d)) for i in att}
        Z = sum(w.values())
        want = [sum(w[i] / Z * V[0, i, c] for i in att) for c in range(d)]
        for out, idx, vals, lse in res:
            assert set(idx[m, 0].tolist()) == set(best)
            np.testing.assert_allclose(out[m, 0], want, rtol=1e-12, atol=1e-14)
            assert abs(lse[m, 0] - (mx / math.sqrt(d) + math.log(Z))) < 1e-12


# ---------------------------------------------------------------- compressed (int8) key index
from oracle import int8_index_ref as i8  # noqa: E402


def test_int8_codes_reconstruct_within_half_a_step():
    g = np.random.default_rng(400)
    x = (g.standard_normal((300, 128)) * g.uniform(0.01, 30.0, (300, 1))).astype(np.float32)
    x[7] = 0.0                                   # an all-zero row
    x[8] = 0.0
    x[8, 5] = 1e-29                              # a row whose largest element is tiny but above the floor
    x[9] = 1e-38                                 # a row below the coding floor of 2^-100: coded as zero
    codes, scale = i8.quantize_rows_int8(x)
    assert codes.dtype == np.int8 and scale.dtype == np.float32
    assert np.abs(codes.astype(np.int32)).max() <= 127
    err = np.abs(x.astype(np.float64) - codes.astype(np.float64) * scale[:, None].astype(np.float64))
    assert (err <= 0.5 * scale[:, None].astype(np.float64) * (1 + 1e-5) + 2.0 ** -100).all()   # floor: rows coded as zero
    # the largest element of every non-zero row is coded +-127, a zero row is all zeros with scale 0
    for r in range(300):
        j = np.abs(x[r]).argmax()
        if abs(x[r, j]) >= 2.0 ** -100:
            assert abs(int(codes[r, j])) == 127 and np.sign(codes[r, j]) == np.sign(x[r, j])
    assert (codes[7] == 0).all() and scale[7] == 0
    assert (codes[9] == 0).all() and scale[9] == 0
    assert codes[8, 5] == 127 and (np.delete(codes[8], 5) == 0).all() and scale[8] > 0
    # odd symmetry and monotonicity within a row
    c2, s2 = i8.quantize_rows_int8(-x)
    assert np.array_equal(c2, -codes) and np.array_equal(s2, scale)
    o = np.argsort(x[3])
    assert (np.diff(codes[3][o].astype(np.int32)) >= 0).all()


def test_int8_codes_agree_with_library_quantiser():
    """torch.quantize_per_tensor with the same scale rounds x * (1/scale) instead of
    x * (127/amax): the two products differ by an ulp at most, so codes may differ only at
    rounding ties, and then by one."""
    g = np.random.default_rng(401)
    x = g.standard_normal((64, 128)).astype(np.float32) * 3
    codes, scale = i8.quantize_rows_int8(x)
    differ = 0
    for r in range(64):
        t = torch.quantize_per_tensor(torch.from_numpy(x[r]), float(scale[r]), 0, torch.qint8).int_repr().numpy()
        d = np.abs(t.astype(np.int32) - codes[r].astype(np.int32))
        assert d.max() <= 1
        differ += int((d != 0).sum())
    assert differ <= 64 * 128 // 200


def test_int8_approx_scores_closed_form_error_bound_and_orientation():
    g = np.random.default_rng(402)
    Hq, Hkv, N, d = 6, 3, 500, 64
    q = g.standard_normal((Hq, d)).astype(np.float32)
    K = g.standard_normal((Hkv, N, d)).astype(np.float32)
    K[1] *= 7.0                                   # a KV head on another scale: catches a wrong head mapping
    A = i8.approx_scores_int8(q, K)
    S = ref.scores(q, K)
    _, sq = i8.quantize_rows_int8(q)
    _, sK = i8.quantize_rows_int8(K)
    for h in range(Hq):
        g_ = h // 2
        # |q.K - q~.K~| <= |q|_1 sK/2 + |K|_1 sq/2 + d sq sK / 4
        bound = (np.abs(q[h]).sum() * sK[g_] / 2 + np.abs(K[g_]).sum(axis=1) * sq[h] / 2 + d * sq[h] * sK[g_] / 4)
        assert (np.abs(A[h] - S[h]) <= bound * (1 + 1e-4)).all()
        # and in practice far tighter: quantisation noise is a few percent of the score spread
        assert np.abs(A[h] - S[h]).std() < 0.05 * S[h].std()
    # integer-valued inputs with amax = 127 are coded exactly: approximate == exact
    qi = g.integers(-127, 128, (2, 32)).astype(np.float32); qi[:, 0] = 127
    Ki = g.integers(-127, 128, (1, 40, 32)).astype(np.float32); Ki[:, :, 1] = -127
    np.testing.assert_array_equal(i8.approx_scores_int8(qi, Ki).astype(np.float64), ref.scores(qi, Ki))


def test_rerank_with_all_candidates_is_the_exact_step_and_recall_grows():
    (qs, Ks, Vs), (q, K, V) = _rand(4, 2, 3000, 32, 403)
    k = 100
    exact = ref.topk_attention(q, K, V, k)
    full = i8.rerank_topk(qs, Ks, Vs, k, 3000)
    np.testing.assert_array_equal(np.sort(full[1], axis=1), np.sort(exact[1], axis=1))
    np.testing.assert_allclose(full[0], exact[0], rtol=1e-12, atol=1e-14)
    prev = 0.0
    for c in (100, 120, 160, 300):
        got = i8.rerank_topk(qs, Ks, Vs, k, c)
        rec = np.mean([i8.recall_at_k(got[1][h], exact[1][h]) for h in range(4)])
        assert rec >= prev - 1e-12
        prev = rec
        # whatever was returned carries its exact score
        for h in range(4):
            np.testing.assert_allclose(got[2][h], (K[h // 2][got[1][h]] @ q[h]), rtol=1e-12)
    assert prev == 1.0            # 3x over-fetch recovers everything at this noise level
    assert i8.recall_at_k(np.array([1, 2, -1]), np.array([2, 3, -1, -1])) == 0.5


# ---------------------------------------------------------------- layer-wise k ("Layer-Wise Settings for k")
# Pins of ref.k_schedule that do not pass through the HIP library: hand-computed shares,
# closed forms and invariants of a fixed-budget largest-remainder split.
def test_k_schedule_hand_computed_cases():
    # uniform budget that divides: every layer the same
    assert ref.k_schedule(32 * 8192, 32, 1.0) == [8192] * 32
    assert ref.k_schedule(77, 1, 9.0) == [77]
    # two layers, last/first = 3: shares 1/4 and 3/4
    assert ref.k_schedule(4000, 2, 3.0) == [1000, 3000]
    # five layers, ratio 3: weights 1, 1.5, 2, 2.5, 3 (sum 10) -> an arithmetic progression
    assert ref.k_schedule(1000, 5, 3.0) == [100, 150, 200, 250, 300]
    # three layers, ratio 3, budget 7: shares 7/6, 14/6, 21/6 -> floors 1, 2, 3; the one key left goes
    # to the largest fractional part (0.5, the last layer)
    assert ref.k_schedule(7, 3, 3.0) == [1, 2, 4]
    # three layers, ratio 2, budget 11: weights 1, 1.5, 2 (sum 4.5) -> shares 2.444, 3.667, 4.889 ->
    # floors 2, 3, 4; two keys left go to fractions 0.889 and 0.667
    assert ref.k_schedule(11, 3, 2.0) == [2, 4, 5]
    # decreasing schedule (ratio 1/2), budget 9, three layers: weights 1, 0.75, 0.5 (sum 2.25) ->
    # shares 4, 3, 2 exactly
    assert ref.k_schedule(9, 3, 0.5) == [4, 3, 2]


def test_k_schedule_ties_go_to_the_later_layer():
    # all fractional parts equal (2.5 each): the two keys left go to the last two layers
    assert ref.k_schedule(10, 4, 1.0) == [2, 2, 3, 3]
    # 100 over 8 layers: 12.5 each, four keys left -> the last four layers
    assert ref.k_schedule(100, 8, 1.0) == [12, 12, 12, 12, 13, 13, 13, 13]
    # ratio 3, two layers, budget 6: shares 1.5 and 4.5 tie at 0.5 -> the later layer is rounded up
    assert ref.k_schedule(6, 2, 3.0) == [1, 5]


@pytest.mark.parametrize("total,L,r", [(262144, 32, 4.0), (1000, 7, 2.5), (33, 32, 8.0), (5000, 3, 0.5),
                                        (32, 32, 5.0), (12345, 17, 1.0), (999, 10, 10.0)])
def test_k_schedule_invariants(total, L, r):
    ks = ref.k_schedule(total, L, r)
    assert len(ks) == L and sum(ks) == total and min(ks) >= 1
    assert all(isinstance(x, int) for x in ks)
    # quota rule of a largest-remainder split: every layer within one key of its exact share
    # (shares below one key are lifted to one, which can only push the others down, never up)
    w = np.array([1.0 + (r - 1.0) * l / (L - 1) if L > 1 else 1.0 for l in range(L)])
    share = total * w / w.sum()
    if share.min() >= 1.0:
        assert (np.abs(np.array(ks) - share) < 1.0 + 1e-9).all()
    else:
        assert (np.array(ks) <= np.maximum(share, 1.0) + 1.0 + 1e-9).all()
    # linear in the layer up to rounding, in the direction the ratio says
    d = np.diff(ks)
    if total >= 8 * L:
        assert (np.abs(np.diff(d)) <= 2).all()
    assert (d >= -1).all() if r >= 1 else (d <= 1).all()


def test_k_schedule_is_monotone_in_the_ratio():
    # a larger last/first ratio moves budget from the first layer to the last
    first, last = [], []
    for r in (1.0, 1.5, 2.0, 3.0, 5.0, 9.0):
        ks = ref.k_schedule(64000, 16, r)
        first.append(ks[0]); last.append(ks[-1])
        assert abs(ks[-1] / ks[0] - r) < 0.01 * r       # the ratio asked for, up to rounding
    assert first == sorted(first, reverse=True) and last == sorted(last)
    # ratio r and 1/r mirror each other (up to which side of a tie is rounded up)
    a, b = ref.k_schedule(64000, 16, 4.0), ref.k_schedule(64000, 16, 0.25)
    assert max(abs(x - y) for x, y in zip(a, b[::-1])) <= 1


# ---------------------------------------------------------------- coarse page index (sub-linear search)
from oracle import page_index_ref as pg


def _pages_case(seed, Hq=4, Hkv=2, N=300, d=16, page=16):
    g = np.random.default_rng(seed)
    q = g.standard_normal((Hq, d))
    K = g.standard_normal((Hkv, N, d)) * g.uniform(0.2, 3.0, (Hkv, N, 1))
    return q, K, page


def test_page_bound_is_never_below_a_key_of_the_page():
    q, K, page = _pages_case(1)
    c, r = pg.page_balls(K, page)
    ub = pg.page_upper_bound(q, c, r)
    S = ref.scores(q, K)
    N = K.shape[1]
    for h in range(q.shape[0]):
        per_key = np.repeat(ub[h], page)[:N]
        assert (S[h] <= per_key + 1e-9).all()
    assert (pg.ball_slack(K, page, c, r) >= -1e-12).all() and np.abs(pg.ball_slack(K, page, c, r)).min() < 1e-12
    assert c.shape == (2, 19, 16) and r.shape == (2, 19)        # 300 tokens: 18 full pages and one of 12


def test_page_bound_is_attained_on_the_sphere_and_is_what_a_minimiser_finds():
    """max of q . x over the ball |x - c| <= r: closed form q . c + |q| r, reached at x = c + r q / |q|; a
    library constrained minimiser (SLSQP on -q . x) finds the same value."""
    from scipy.optimize import minimize
    g = np.random.default_rng(2)
    d = 6
    for _ in range(5):
        q, c, r = g.standard_normal(d), g.standard_normal(d), float(g.uniform(0.1, 2.0))
        ub = pg.page_upper_bound(q[None], c[None, None], np.array([[r]]))[0, 0]
        x_star = c + r * q / np.linalg.norm(q)
        assert abs(q @ x_star - ub) < 1e-12
        res = minimize(lambda x: -(q @ x), c, constraints=[{"type": "ineq", "fun": lambda x: r * r - (x - c) @ (x - c)}],
                       method="SLSQP", options={"ftol": 1e-12, "maxiter": 500})
        assert abs(-res.fun - ub) < 1e-5
    # a key placed on that point makes the bound tight for its page
    K = np.stack([c + 0.1 * g.standard_normal(d) for _ in range(7)] )[None]
    cc, rr = pg.page_balls(K, 8)
    far = cc[0, 0] + rr[0, 0] * q / np.linalg.norm(q)
    assert abs(pg.page_upper_bound(q[None], cc, rr)[0, 0] - q @ far) < 1e-12


def test_page_bound_special_cases():
    g = np.random.default_rng(3)
    q = g.standard_normal((2, 8))
    row = g.standard_normal(8)
    K = np.tile(row, (1, 32, 1))                              # identical keys: radius 0, bound = the score
    c, r = pg.page_balls(K, 8)
    assert np.abs(r).max() < 1e-12
    np.testing.assert_allclose(pg.page_upper_bound(q, c, r), np.tile((q @ row)[:, None], (1, 4)), rtol=1e-12)
    # two keys: the centre is their midpoint, the radius half their distance
    K2 = np.stack([row, row + 2.0])[None]
    c2, r2 = pg.page_balls(K2, 2)
    np.testing.assert_allclose(c2[0, 0], row + 1.0)
    assert abs(r2[0, 0] - np.sqrt(8.0)) < 1e-12
    # linear in beta between the centre's score and the full bound
    q3, K3, page = _pages_case(4)
    c3, r3 = pg.page_balls(K3, page)
    b0, b1, bh = (pg.page_upper_bound(q3, c3, r3, b) for b in (0.0, 1.0, 0.5))
    np.testing.assert_allclose(bh, 0.5 * (b0 + b1), rtol=1e-12)
    np.testing.assert_allclose(b0[1], c3[0] @ q3[1], rtol=1e-12)     # head 1 reads KV head 0 (G = 2)
    np.testing.assert_allclose(b0[2], c3[1] @ q3[2], rtol=1e-12)     # head 2 reads KV head 1
    assert (b1 >= b0).all()


def test_pages_an_exact_search_must_read_and_restricted_search():
    q, K, page = _pages_case(5, N=257)
    S = ref.scores(q, K)
    k, G = 20, 2
    c, r = pg.page_balls(K, page)
    ub = pg.page_upper_bound(q, c, r)
    idx = np.stack([ref.select_topk(S[h], k)[0] for h in range(4)])
    need = pg.pages_holding_topk(idx, c.shape[1], page, G)
    # brute force: a page is needed iff removing it changes some head's selection
    for g_ in range(2):
        for p in range(c.shape[1]):
            hit = any(((idx[h] // page) == p).any() for h in (2 * g_, 2 * g_ + 1))
            assert need[g_, p] == hit
    s_k = np.array([np.sort(S[h])[::-1][k - 1] for h in range(4)])
    for level in (s_k, s_k - 0.5, np.full(4, -np.inf)):
        keep = pg.pages_above(ub, level, G)
        assert (keep | ~need).all()                           # every needed page is kept at a cut-off <= the k-th score
        got = pg.search_in_pages(S, keep, k, page, G)
        for h in range(4):
            np.testing.assert_array_equal(got[h], idx[h])     # and the restricted search is the exact one
    assert pg.pages_above(ub, np.full(4, -np.inf), G).all()
    # a cut-off above the k-th score may lose keys: then the restricted search differs (the approximate regime)
    keep_hi = pg.pages_above(ub, ub.max(axis=1) - 1e-9, G)   # only each head's best-looking page survives
    assert keep_hi.sum() <= 4 and not (keep_hi | ~need).all()
    # pages_above takes the union over the heads of a group
    solo = ub >= s_k[:, None]
    np.testing.assert_array_equal(pg.pages_above(ub, s_k, G), solo[0::2] | solo[1::2])
