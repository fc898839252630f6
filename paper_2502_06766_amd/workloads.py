"""Seeded synthetic KV caches and queries for top-k attention decode.

This module only draws random numbers and shapes them into caches whose
statistics resemble the long-context decode workloads the method targets
(a query that is strongly aligned with a small set of cached keys, a few
high-magnitude channels, attention mass concentrated on ~2 % of positions).
It contains none of the method's arithmetic (no scoring, selection or
softmax): both the CPU oracle and the HIP path consume exactly the arrays it
returns, rounded to the storage dtype.

Random streams are counter based (Philox) and keyed by
(seed, config id, layer * n_seqs + seq, kv_head), so any slice of a workload
can be regenerated on its own and the kv heads can be filled by independent
host threads.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

F32, F16, BF16 = 0, 1, 2  # storage dtype codes (same values as the C-ABI enum)
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}
DTYPE_BYTES = {F32: 4, F16: 2, BF16: 2}


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape of one synthetic decode workload."""
    name: str
    config_id: int
    n_layers: int
    n_seqs: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_tokens: int
    k: int
    dtype: int
    recipe: str          # "planted_sum" | "planted_cos" | "score_shaped" | "clustered"
    n_planted: int = 0   # per query head (planted_cos) or in total (planted_sum)
    n_outlier_channels: int = 0

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def scaled(self, n_tokens: int, k: Optional[int] = None, **kw) -> "Workload":
        """Same recipe at another context length (used for parity sweeps)."""
        if k is None:
            k = max(1, int(round(self.k * n_tokens / self.n_tokens)))
        return dataclasses.replace(self, n_tokens=n_tokens, k=k, **kw)


# The five benchmark configurations (synthetic stand-ins for Llama-3-8B KV
# caches on long-context retrieval prompts; see the recipes below).
C1 = Workload("c1_single_head_fp32", 1, 1, 1, 1, 1, 64, 4096, 64, F32,
              "planted_sum", n_planted=4)
C2 = Workload("c2_llama8b_layer_128k_bf16", 2, 1, 1, 32, 8, 128, 131072, 2048, BF16,
              "planted_cos", n_planted=64, n_outlier_channels=4)
C3 = Workload("c3_llama8b_layer_1m_fp16", 3, 1, 1, 32, 8, 128, 1048576, 16384, F16,
              "planted_cos", n_planted=64, n_outlier_channels=4)
C4 = Workload("c4_batched16_256k_bf16", 4, 1, 16, 32, 8, 128, 262144, 1024, BF16,
              "planted_cos", n_planted=64, n_outlier_channels=4)
C5 = Workload("c5_32layer_512k_fp16", 5, 32, 1, 32, 8, 128, 524288, 8192, F16,
              "score_shaped")
# Not one of the five: a cache with the structure that lets a coarse index rule out whole pages (see
# make_clustered), for the sub-linear search.
C6 = Workload("c6_clustered_1m_fp16", 6, 1, 1, 32, 8, 128, 1048576, 16384, F16, "clustered")
CONFIGS = {w.config_id: w for w in (C1, C2, C3, C4, C5)}
C4_K_SWEEP = (256, 1024, 4096)

# c5: score offset that puts ~95 % of the dense softmax mass on a random 2 %
# of positions: ln(0.95 * 0.98 / (0.05 * 0.02)).
C5_HOT_FRACTION = 0.02
C5_DELTA = float(np.log(0.95 * 0.98 / (0.05 * 0.02)))


def _rng(seed: int, config_id: int, unit: int, stream: int) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(32)) | np.uint64(config_id & 0xFFFFFFFF)
    ctr = (np.uint64(unit) << np.uint64(32)) | np.uint64(stream & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=[key, ctr]))


# --------------------------------------------------------------------------
# storage-dtype rounding (data preparation only)
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round a float32 array to the storage dtype.

    Returns float32 for F32, float16 for F16 and uint16 bfloat16 bit patterns
    for BF16 (numpy has no bfloat16).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F32:
        return x
    if dtype == F16:
        return x.astype(np.float16)
    if dtype == BF16:
        return to_bf16_bits(x)
    raise ValueError(f"unknown dtype code {dtype}")


def widen(xq: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> float64 holding exactly the stored values."""
    if dtype == BF16:
        return bf16_bits_to_f32(xq).astype(np.float64)
    return xq.astype(np.float64)


def storage_numpy_dtype(dtype: int):
    return {F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype]


# --------------------------------------------------------------------------
# recipes
# --------------------------------------------------------------------------
def make_query(w: Workload, seed: int, layer: int = 0, seq: int = 0) -> np.ndarray:
    """Pre-quantisation query block [Hq, d] float32 for recipes whose query does
    not depend on the cache (planted_cos, score_shaped)."""
    g = _rng(seed, w.config_id, layer * w.n_seqs + seq, 0x7FFF0000)
    return g.standard_normal((w.n_q_heads, w.head_dim), dtype=np.float32)


def _fill_head_planted_cos(w, seed, layer, seq, h_kv, q, K, V):
    unit = layer * w.n_seqs + seq
    g = _rng(seed, w.config_id, unit, h_kv)
    N, d, G = w.n_tokens, w.head_dim, w.group
    g.standard_normal(out=K[h_kv], dtype=np.float32)
    g.standard_normal(out=V[h_kv], dtype=np.float32)
    if w.n_outlier_channels:
        ch = g.choice(d, size=w.n_outlier_channels, replace=False)
        K[h_kv][:, ch] *= 8.0
        V[h_kv][:, ch] *= 8.0
    n_pl = min(w.n_planted, N // (2 * G))
    if n_pl > 0:
        pos = g.choice(N, size=n_pl * G, replace=False).reshape(G, n_pl)
        for j in range(G):
            qh = q[h_kv * G + j].astype(np.float64)
            qhat = qh / np.linalg.norm(qh)
            rows = K[h_kv][pos[j]].astype(np.float64)
            norms = np.linalg.norm(rows, axis=1, keepdims=True)
            nz = g.standard_normal((n_pl, d))
            nz -= (nz @ qhat)[:, None] * qhat[None, :]
            nz /= np.linalg.norm(nz, axis=1, keepdims=True)
            K[h_kv][pos[j]] = (norms * (0.6 * qhat[None, :] + 0.8 * nz)).astype(np.float32)


def _fill_head_score_shaped(w, seed, layer, seq, h_kv, q, K, V):
    """Keys built so that the G queries of the group see prescribed scores:
    K_i = Q^+ t_i + (I - Q^+ Q) n_i  with  t_{h,i} = sqrt(d) (z + Delta [i in hot_h])."""
    unit = layer * w.n_seqs + seq
    g = _rng(seed, w.config_id, unit, h_kv)
    N, d, G = w.n_tokens, w.head_dim, w.group
    Q = q[h_kv * G:(h_kv + 1) * G].astype(np.float64)        # [G, d]
    Qp = np.linalg.pinv(Q)                                    # [d, G]
    P = np.eye(d) - Qp @ Q                                    # null-space projector
    g.standard_normal(out=V[h_kv], dtype=np.float32)
    n_hot = max(1, int(round(C5_HOT_FRACTION * N)))
    blk = 65536
    hot = np.zeros((G, N), dtype=bool)
    for j in range(G):
        hot[j, g.choice(N, size=n_hot, replace=False)] = True
    for s in range(0, N, blk):
        e = min(N, s + blk)
        z = g.standard_normal((e - s, G))
        t = np.sqrt(d) * (z + C5_DELTA * hot[:, s:e].T)       # [n, G]
        n = g.standard_normal((e - s, d))
        K[h_kv][s:e] = (t @ Qp.T + n @ P.T).astype(np.float32)


# c6: topical runs.  Every KV head draws N_CENTROIDS centroids ~ N(0, 1); the sequence is a chain of runs of
# CLUSTER_RUN[0] .. CLUSTER_RUN[1] consecutive tokens, each run around one centroid (picked at random), its
# keys the centroid plus N(0, sigma^2) noise.  A query head is Gaussian plus CLUSTER_PULL times the sum of
# CLUSTER_HOT centroids of its KV head, so the keys it attends to sit in the runs of a few centroids, while
# the other runs score like unrelated text.  `sigma` is how tight a run is: the page index can rule a page
# out only if its keys are close together.
N_CENTROIDS = 256
CLUSTER_RUN = (128, 2048)
CLUSTER_HOT = 3
CLUSTER_PULL = 0.25
CLUSTER_SIGMA = 0.02


def _cluster_rng(w, seed, layer, seq, h_kv):
    return _rng(seed, w.config_id, layer * w.n_seqs + seq, 0x10000 + h_kv)


def _cluster_centroids(w, seed, layer, seq, h_kv):
    g = _rng(seed, w.config_id, layer * w.n_seqs + seq, 0x20000 + h_kv)
    return g.standard_normal((N_CENTROIDS, w.head_dim), dtype=np.float32)


def _fill_head_clustered(w, seed, layer, seq, h_kv, q, K, V, sigma):
    g = _cluster_rng(w, seed, layer, seq, h_kv)
    N, d = w.n_tokens, w.head_dim
    C = _cluster_centroids(w, seed, layer, seq, h_kv)
    g.standard_normal(out=K[h_kv], dtype=np.float32)
    g.standard_normal(out=V[h_kv], dtype=np.float32)
    K[h_kv] *= np.float32(sigma)
    pos = 0
    while pos < N:
        run = int(g.integers(CLUSTER_RUN[0], CLUSTER_RUN[1] + 1))
        K[h_kv][pos:pos + run] += C[int(g.integers(N_CENTROIDS))]
        pos += run


def make_clustered(w: Workload, seed: int, sigma: float = CLUSTER_SIGMA, layer: int = 0, seq: int = 0, threads: int = 8):
    """(q, K, V) float32 of the clustered recipe (see above), before rounding to the storage dtype."""
    N, d, G = w.n_tokens, w.head_dim, w.group
    K = np.empty((w.n_kv_heads, N, d), dtype=np.float32)
    V = np.empty((w.n_kv_heads, N, d), dtype=np.float32)
    q = make_query(w, seed, layer, seq)
    for h in range(w.n_q_heads):
        gq = _rng(seed, w.config_id, layer * w.n_seqs + seq, 0x30000 + h)
        hot = gq.choice(N_CENTROIDS, size=CLUSTER_HOT, replace=False)
        q[h] += np.float32(CLUSTER_PULL) * _cluster_centroids(w, seed, layer, seq, h // G)[hot].sum(axis=0)
    if threads > 1 and w.n_kv_heads > 1 and N * d >= (1 << 22):
        with ThreadPoolExecutor(max_workers=min(threads, w.n_kv_heads)) as ex:
            list(ex.map(lambda h: _fill_head_clustered(w, seed, layer, seq, h, q, K, V, sigma), range(w.n_kv_heads)))
    else:
        for h in range(w.n_kv_heads):
            _fill_head_clustered(w, seed, layer, seq, h, q, K, V, sigma)
    return q, K, V


def make_cache(w: Workload, seed: int, layer: int = 0, seq: int = 0, threads: int = 8):
    """Returns (q [Hq,d], K [Hkv,N,d], V [Hkv,N,d]) as float32, before rounding
    to the storage dtype."""
    N, d = w.n_tokens, w.head_dim
    K = np.empty((w.n_kv_heads, N, d), dtype=np.float32)
    V = np.empty((w.n_kv_heads, N, d), dtype=np.float32)
    if w.recipe == "clustered":
        return make_clustered(w, seed, CLUSTER_SIGMA, layer, seq, threads)
    if w.recipe == "planted_sum":
        assert w.n_q_heads == 1 and w.n_kv_heads == 1
        g = _rng(seed, w.config_id, layer * w.n_seqs + seq, 0)
        g.standard_normal(out=K[0], dtype=np.float32)
        g.standard_normal(out=V[0], dtype=np.float32)
        planted = g.choice(N, size=min(w.n_planted, N), replace=False)
        noise = 0.1 * g.standard_normal(d, dtype=np.float32)
        q = (K[0][planted].sum(axis=0) + noise)[None, :].astype(np.float32)
        return q, K, V
    q = make_query(w, seed, layer, seq)
    fill = {"planted_cos": _fill_head_planted_cos,
            "score_shaped": _fill_head_score_shaped}[w.recipe]
    if threads > 1 and w.n_kv_heads > 1 and N * d >= (1 << 22):
        with ThreadPoolExecutor(max_workers=min(threads, w.n_kv_heads)) as ex:
            list(ex.map(lambda h: fill(w, seed, layer, seq, h, q, K, V), range(w.n_kv_heads)))
    else:
        for h in range(w.n_kv_heads):
            fill(w, seed, layer, seq, h, q, K, V)
    return q, K, V


def make_quantized(w: Workload, seed: int, layer: int = 0, seq: int = 0, threads: int = 8):
    """(q, K, V) rounded to the workload's storage dtype (see `quantize`)."""
    q, K, V = make_cache(w, seed, layer, seq, threads)
    return quantize(q, w.dtype), quantize(K, w.dtype), quantize(V, w.dtype)


def make_query_chunk(q: np.ndarray, dtype: int, n_queries: int, seed: int, rho: float = 0.8) -> np.ndarray:
    """A chunk of consecutive queries [M, Hq, d] (storage dtype) whose last row is the
    given query block q [Hq, d] (storage dtype): neighbouring tokens ask for similar
    things, so row m is q mixed with fresh noise of the same per-head norm, with
    correlation rho ** (M - 1 - m) to q."""
    qf = bf16_bits_to_f32(q) if dtype == BF16 else q.astype(np.float32)
    Hq, d = qf.shape
    g = _rng(seed, 0x51C0FFEE, n_queries, 0x7FFE0000)
    norm = np.linalg.norm(qf, axis=1, keepdims=True)
    rows = []
    for m in range(n_queries):
        c = rho ** (n_queries - 1 - m)
        noise = g.standard_normal((Hq, d), dtype=np.float32)
        noise *= norm / np.maximum(np.linalg.norm(noise, axis=1, keepdims=True), 1e-20)
        rows.append(qf if m == n_queries - 1 else (c * qf + np.sqrt(1.0 - c * c) * noise).astype(np.float32))
    out = quantize(np.stack(rows), dtype)
    out[n_queries - 1] = q
    return out


def kv_cache_bytes(n_tokens: int, hidden: int, n_layers: int, bytes_per_el: int) -> int:
    """Size of a dense KV cache: two tensors of n_tokens x hidden per layer."""
    return 2 * n_tokens * hidden * n_layers * bytes_per_el
