"""The seeded input generators: every input is synthetic, and the structure stated for
each configuration (planted keys, outlier channels, concentrated softmax mass, the length
and head shapes) is checked here on scaled-down instances, together with the storage
rounding helpers the tests and the benchmark share."""
import numpy as np
import pytest

from paper_2502_06766_amd import workloads as wl


def test_configs_have_the_stated_shapes():
    c = wl.CONFIGS
    assert (c[1].n_q_heads, c[1].n_kv_heads, c[1].head_dim, c[1].n_tokens, c[1].k, c[1].dtype) == \
        (1, 1, 64, 4096, 64, wl.F32)
    assert (c[2].n_q_heads, c[2].n_kv_heads, c[2].head_dim, c[2].n_tokens, c[2].k, c[2].dtype) == \
        (32, 8, 128, 131072, 2048, wl.BF16)
    assert (c[3].n_q_heads, c[3].n_kv_heads, c[3].head_dim, c[3].n_tokens, c[3].k, c[3].dtype) == \
        (32, 8, 128, 1048576, 16384, wl.F16)
    assert (c[4].n_seqs, c[4].n_tokens, c[4].dtype) == (16, 262144, wl.BF16) and wl.C4_K_SWEEP == (256, 1024, 4096)
    assert (c[5].n_layers, c[5].n_tokens, c[5].k, c[5].dtype) == (32, 524288, 8192, wl.F16)
    # c5: about 64 GB of K and V in 16 bit
    assert 2 * c[5].n_layers * c[5].n_kv_heads * c[5].n_tokens * c[5].head_dim * 2 == 64 * 2 ** 30


def test_same_seed_same_bytes_other_seed_other_bytes():
    w = wl.C2.scaled(4096)
    a = wl.make_quantized(w, 5)
    b = wl.make_quantized(w, 5, threads=1)
    c = wl.make_quantized(w, 6)
    d = wl.make_quantized(w, 5, layer=1)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    assert not np.array_equal(a[1], c[1]) and not np.array_equal(a[0], c[0])
    assert not np.array_equal(a[1], d[1])


def test_c1_query_is_the_sum_of_its_planted_keys():
    q, K, V = wl.make_cache(wl.C1, 0)
    assert q.shape == (1, 64) and K.shape == (1, 4096, 64)
    s = K[0].astype(np.float64) @ q[0].astype(np.float64)
    # a planted key scores about |key|^2 = 64 (+- 14), the others N(0, 4 * 64): all four are among the
    # best 16, and q is their plain sum up to the recipe's N(0, 0.1) noise
    top = np.argsort(-s)[:16]
    coef, *_ = np.linalg.lstsq(K[0][top].astype(np.float64).T, q[0].astype(np.float64), rcond=None)
    planted = top[np.abs(coef - 1.0) < 0.05]
    assert planted.size == 4 and (np.abs(np.delete(coef, np.flatnonzero(np.abs(coef - 1.0) < 0.05))) < 0.05).all()
    resid = q[0] - K[0][planted].sum(axis=0)
    assert 0.06 < resid.std() < 0.15
    assert set(planted.tolist()) <= set(np.argsort(-s)[:wl.C1.k].tolist())


def test_c2_recipe_outlier_channels_and_planted_cosine():
    w = wl.C2.scaled(8192)
    q, K, V = wl.make_cache(w, 1)
    for h in range(w.n_kv_heads):
        std = K[h].std(axis=0)
        big = np.sort(std)[-4:]
        rest = np.sort(std)[:-4]
        assert (big > 6.0).all() and (rest < 1.5).all()           # four channels scaled by 8
        assert (np.sort(V[h].std(axis=0))[-4:] > 6.0).all()
    # every query head has 64 keys at cosine 0.6 (far outside what random keys reach)
    G = w.group
    for hq in (0, 5, 31):
        kh = K[hq // G].astype(np.float64)
        qv = q[hq].astype(np.float64)
        cos = kh @ qv / (np.linalg.norm(kh, axis=1) * np.linalg.norm(qv))
        top = np.sort(cos)[::-1]
        assert np.allclose(top[:64], 0.6, atol=1e-3)
        assert top[64 + 3 * 64] < 0.5        # the other heads' planted keys are not aligned with this one


def test_c5_recipe_concentrates_the_softmax_mass():
    w = wl.C5.scaled(16384, k=328, n_layers=1)
    q, K, V = wl.make_cache(w, 2)
    d = w.head_dim
    for hq in (0, 9, 31):
        s = K[hq // w.group].astype(np.float64) @ q[hq].astype(np.float64) / np.sqrt(d)
        p = np.exp(s - s.max())
        p /= p.sum()
        top2 = np.sort(p)[::-1][:int(round(0.02 * w.n_tokens))].sum()
        assert 0.90 < top2 < 0.985           # about 95 % of the mass on the top 2 % of the keys


def test_query_chunk_correlation_and_last_row():
    w = wl.C3.scaled(256)
    q = wl.make_quantized(w, 0)[0]
    ch = wl.make_query_chunk(q, w.dtype, 5, 3, rho=0.8)
    assert ch.shape == (5,) + q.shape and ch.dtype == q.dtype
    assert np.array_equal(ch[-1], q)
    qf = q.astype(np.float64)
    for m in range(4):
        row = ch[m].astype(np.float64)
        cos = (row * qf).sum(axis=1) / (np.linalg.norm(row, axis=1) * np.linalg.norm(qf, axis=1))
        assert abs(np.median(cos) - 0.8 ** (4 - m)) < 0.08
        assert np.allclose(np.linalg.norm(row, axis=1), np.linalg.norm(qf, axis=1), rtol=0.15)


@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_quantize_is_idempotent_and_widen_exact(dtype):
    g = np.random.default_rng(0)
    x = (g.standard_normal(4096) * np.exp(g.uniform(-20, 9, 4096))).astype(np.float32)      # inside fp16 range
    xq = wl.quantize(x, dtype)
    assert xq.dtype == wl.storage_numpy_dtype(dtype)
    back = wl.widen(xq, dtype)
    assert back.dtype == np.float64
    again = wl.quantize(back.astype(np.float32), dtype)
    assert np.array_equal(again, xq)
    rel = {wl.F32: 0.0, wl.F16: 2.0 ** -11, wl.BF16: 2.0 ** -8}[dtype]
    ok = np.abs(x) > 1e-4 if dtype == wl.F16 else np.ones_like(x, dtype=bool)      # fp16 subnormals aside
    ok &= np.abs(x) < 6e4
    assert (np.abs(back[ok] - x[ok]) <= rel * np.abs(x[ok]) * 1.0001).all()


def test_bf16_rounds_to_nearest_even():
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: ties go to the even mantissa
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = wl.bf16_bits_to_f32(wl.to_bf16_bits(x))
    assert got.tolist() == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7]


def test_clustered_recipe_has_runs_a_page_index_can_rule_out():
    """c6: keys in runs around a few hundred centroids.  Seeded and repeatable; the tighter the runs the
    fewer pages hold a score bound that reaches the k-th score (figures from the float64 oracle)."""
    from oracle import page_index_ref as pg
    from oracle import topk_attention_ref as ref
    w = wl.C6.scaled(32768)
    a = wl.make_clustered(w, 3, 0.05)
    b = wl.make_clustered(w, 3, 0.05)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)
    assert not np.array_equal(wl.make_clustered(w, 4, 0.05)[1], a[1])
    q0, K0, _ = wl.make_cache(w, 3)                               # the recipe's default tightness
    np.testing.assert_array_equal(K0, wl.make_clustered(w, 3, wl.CLUSTER_SIGMA)[1])
    kept = []
    for sigma in (0.02, 0.1, 0.4):
        q, K, V = wl.make_clustered(w, 3, sigma)
        qd, Kd = wl.widen(wl.quantize(q, w.dtype), w.dtype), wl.widen(wl.quantize(K, w.dtype), w.dtype)
        S = ref.scores(qd, Kd)
        c, r = pg.page_balls(Kd, 64)
        s_k = np.sort(S, axis=1)[:, -w.k]
        kept.append(pg.pages_above(pg.page_upper_bound(qd, c, r), s_k, w.group).mean())
        # within a run the keys stay close to their centroid: the median page radius is about sigma sqrt(d)
        assert 0.7 * sigma * np.sqrt(w.head_dim) < np.median(r) < 1.6 * sigma * np.sqrt(w.head_dim)
    assert kept[0] < 0.35 and kept[0] < kept[1] < kept[2] and kept[2] > 0.95
