"""CPU oracle for top-k attention decode (NumPy, float64).  TEST INFRASTRUCTURE.

This file is the plain definition of what the decode path computes, written
from the paper's methodology section ("Top-k Attention: Accelerating
Decoding") and its decoding algorithm (Algorithm 1, the search step and the
attention step over the selected rows).  It is slow on purpose: full score
vector, full sort, double precision.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path never does, and
this file shares no code with the HIP kernels.

Conventions (readings of the paper where it is silent are listed in the
design notes):
  * one key/value stream per KV head; query head h searches KV head h // G with
    G = n_q_heads // n_kv_heads, and every query head selects its own top-k;
  * the search metric is the raw dot product q . K_i (the paper's "dot product
    metric"); the 1/sqrt(d) scale of Eq. 1 is applied inside the softmax, with
    d the per-head dimension;
  * ties are broken towards the lower position;
  * k_eff = min(k, N); unused output slots hold index -1 / value -inf.

Pins: every function here is pinned by tests/test_oracle_pins.py (k = N equals
library dense attention, brute-force subset enumeration on tiny N, k = 1,
all-equal scores, score-shift invariance, permutation invariance, planted
dominant keys, truncation-error bound; for the window variant: window 0 equals the
plain step, full coverage equals library dense attention, brute force on tiny N, and
the log-sum-exp merge of a top-k prefix with library attention over the window;
for the multi-query variant: k >= N with a causal chunk equals library causal dense
attention, the last causal query equals the plain step, and brute force on tiny N;
for k_schedule: hand-computed shares including ties in the fractional parts, closed forms
(uniform split, two-layer ratio, arithmetic progression), sum = budget, every layer >= 1,
the quota rule and monotonicity in the ratio).
No function is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def scores(q: np.ndarray, K: np.ndarray) -> np.ndarray:
    """Score matrix S = q K^T of Eq. 1, one row per query head.

    q [Hq, d], K [Hkv, N, d] (float64 holding the stored values) -> [Hq, N].
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    Hq, d = q.shape
    Hkv, N, dk = K.shape
    assert d == dk and Hq % Hkv == 0
    G = Hq // Hkv
    S = np.empty((Hq, N), dtype=np.float64)
    for h in range(Hq):
        S[h] = K[h // G] @ q[h]
    return S


def select_topk(s: np.ndarray, k: int):
    """The exact k-nearest-neighbour search of the methodology section for one
    query head under the dot-product metric: full sort of (score descending,
    position ascending), keep the first min(k, N).

    s [N] -> (I [k_eff] int64, vals [k_eff] float64), in sorted order.
    """
    s = np.asarray(s, dtype=np.float64)
    N = s.shape[0]
    k_eff = min(int(k), N)
    order = np.lexsort((np.arange(N), -s))   # primary key -s, secondary position
    I = order[:k_eff]
    return I.astype(np.int64), s[I]


def attend_selected(vals: np.ndarray, Vsel: np.ndarray, d: int):
    """Attention step of Algorithm 1 over the retrieved rows:
    Softmax(vals / sqrt(d)) V[I], max-subtracted.

    vals [k], Vsel [k, d] -> (out [d], lse) with lse the log-sum-exp of the
    scaled selected scores.
    """
    z = np.asarray(vals, dtype=np.float64) / np.sqrt(float(d))
    m = z.max()
    w = np.exp(z - m)
    Z = w.sum()
    p = w / Z
    out = p @ np.asarray(Vsel, dtype=np.float64)
    return out, float(m + np.log(Z))


def topk_attention(q, K, V, k: int):
    """Whole decode step for one (layer, sequence).

    q [Hq, d], K, V [Hkv, N, d] float64 (already rounded to the storage dtype)
    -> out [Hq, d] f64, idx [Hq, k] int64 (-1 padded), vals [Hq, k] f64
       (-inf padded), lse [Hq] f64.  idx/vals rows are in descending score order.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    if k < 1 or N < 1:
        raise ValueError("k and N must be >= 1")
    S = scores(q, K)
    out = np.zeros((Hq, d))
    idx = np.full((Hq, k), -1, dtype=np.int64)
    vals = np.full((Hq, k), -np.inf)
    lse = np.zeros(Hq)
    for h in range(Hq):
        I, v = select_topk(S[h], k)
        ke = I.shape[0]
        idx[h, :ke] = I
        vals[h, :ke] = v
        out[h], lse[h] = attend_selected(v, V[h // G][I], d)
    return out, idx, vals, lse


def topk_attention_window(q, K, V, k: int, window: int):
    """Decode step with the recent-token window of Algorithm 1: the last `window`
    cached tokens play the role of K_gen / V_gen (always attended), the k-nearest-
    neighbour search runs over the older prefix only, and one softmax spans the
    retrieved scores and the window scores together (the reading taken for the
    algorithm's window line, whose printed form lacks the value factor).

    Returns out [Hq, d], idx [Hq, k] (search result over the prefix, -1 padded),
    vals [Hq, k] (-inf padded), lse [Hq] (over retrieved + window scores).
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    if k < 1 or N < 1 or window < 0:
        raise ValueError("k, N must be >= 1 and window >= 0")
    W = min(int(window), N)
    P = N - W                               # the search runs over positions [0, P)
    S = scores(q, K)
    out = np.zeros((Hq, d))
    idx = np.full((Hq, k), -1, dtype=np.int64)
    vals = np.full((Hq, k), -np.inf)
    lse = np.zeros(Hq)
    for h in range(Hq):
        if P > 0:
            I, v = select_topk(S[h, :P], k)
        else:
            I, v = np.zeros(0, dtype=np.int64), np.zeros(0)
        idx[h, :I.shape[0]] = I
        vals[h, :I.shape[0]] = v
        rows = np.concatenate([I, np.arange(P, N)])          # retrieved positions, then the window
        out[h], lse[h] = attend_selected(S[h, rows], V[h // G][rows], d)
    return out, idx, vals, lse


def topk_attention_multi(q, K, V, k: int, causal: bool, window: int = 0):
    """A chunk of M queries against one cache, each an independent decode step (the
    multi-query use of top-k attention: the paper notes that top-k can also serve while
    the cache is built, in the section on generating million-token caches).

    q [M, Hq, d].  With `causal` the queries are those of the last M cached tokens and
    query m sees the first N - (M - 1 - m) tokens only (itself and everything before);
    otherwise all queries see all N.  Returns out [M, Hq, d], idx, vals [M, Hq, k],
    lse [M, Hq]: row m is topk_attention_window on the visible part of the cache.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    M = q.shape[0]
    N = K.shape[1]
    res = []
    for m in range(M):
        n_vis = N - (M - 1 - m) if causal else N
        if n_vis < 1:
            raise ValueError("a causal chunk needs at least M cached tokens")
        res.append(topk_attention_window(q[m], K[:, :n_vis], V[:, :n_vis], k, window))
    return tuple(np.stack([r[i] for r in res]) for i in range(4))


def attention_entropy(s: np.ndarray, d: int) -> float:
    """Shannon entropy E = -sum a_i log a_i of the softmaxed score row
    (the paper's sparsity diagnostic); its maximum is log N."""
    z = np.asarray(s, dtype=np.float64) / np.sqrt(float(d))
    z = z - z.max()
    a = np.exp(z)
    a /= a.sum()
    nz = a > 0
    return float(-(a[nz] * np.log(a[nz])).sum())


def captured_mass(s: np.ndarray, I: np.ndarray, d: int) -> float:
    """Share of the dense softmax mass carried by the positions I."""
    z = np.asarray(s, dtype=np.float64) / np.sqrt(float(d))
    z = z - z.max()
    a = np.exp(z)
    return float(a[I].sum() / a.sum())


def k_schedule(total_k: int, n_layers: int, last_over_first: float = 1.0):
    """Layer-wise k of the paper's "Layer-Wise Settings for k": a fixed total budget
    sum_l k_l, uniform (ratio 1) or increasing linearly from the first to the last layer.
    Exact rational shares total_k * w_l / sum(w), w_l = 1 + (ratio - 1) l / (L - 1), rounded
    by largest remainder (later layer first on ties), every layer at least 1."""
    from fractions import Fraction
    L = n_layers
    r = Fraction(last_over_first).limit_denominator(1 << 20)
    w = [Fraction(1) if L == 1 else 1 + (r - 1) * Fraction(l, L - 1) for l in range(L)]
    tot = sum(w)
    exact = [total_k * x / tot for x in w]
    k = [max(1, int(e)) for e in exact]          # int() floors positive fractions
    order = sorted(range(L), key=lambda l: (exact[l] - k[l], l), reverse=True)
    rem = total_k - sum(k)
    i = 0
    while rem > 0:
        k[order[i % L]] += 1
        rem -= 1
        i += 1
    i = L - 1
    while rem < 0:
        if k[order[i % L]] > 1:
            k[order[i % L]] -= 1
            rem += 1
        i -= 1
    return k
