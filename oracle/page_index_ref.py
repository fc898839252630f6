"""CPU oracle for the coarse page index of the sub-linear search (NumPy, float64).  TEST INFRASTRUCTURE.

The methodology section of the paper leaves the search index open; the point of the method is that
the k best keys of a query can be found without reading every key (the sub-linear search its
introduction aims at).  The index here is a plain one that lets whole groups of keys be ruled out exactly:
the cache is cut into pages of `page` consecutive tokens, and each page keeps a centre c (the mean of
its keys) and a radius r (the largest Euclidean distance of one of its keys from the centre).  By the
Cauchy-Schwarz inequality no key of the page can score more than

    UB(q, page) = q . c + |q| r,

so a page whose bound is below a score that k keys are known to reach cannot hold any of the k best
keys and need not be read.  With `beta` < 1 the radius is shrunk (bound = q . c + beta |q| r): fewer
pages are read and keys may be missed (approximate search, judged by recall against the exact one).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file; it shares no
code with the HIP kernels.  Pins (tests/test_oracle_pins.py): the bound is never below the score of a
key of its page, is attained by a key that lies on the sphere in the direction of q, equals the score
for a page of identical keys, is what a library minimiser finds for the maximum of q . x over the
ball, and is linear in beta; the pages an exact search must read are those that hold one of the k
best keys (brute force), and a search restricted to the pages kept at any cut-off not above the k-th
score returns exactly the k best keys.
"""
from __future__ import annotations

import numpy as np


def page_balls(K: np.ndarray, page: int):
    """K [Hkv, N, d] -> (centre [Hkv, P, d], radius [Hkv, P]) with P = ceil(N / page): the mean of the
    keys of each page (the last page may be partial) and the largest distance of a key from it."""
    K = np.asarray(K, dtype=np.float64)
    Hkv, N, d = K.shape
    P = (N + page - 1) // page
    centre = np.empty((Hkv, P, d))
    radius = np.empty((Hkv, P))
    for p in range(P):
        rows = K[:, p * page:min(N, (p + 1) * page)]
        centre[:, p] = rows.mean(axis=1)
        radius[:, p] = np.sqrt(((rows - centre[:, p][:, None, :]) ** 2).sum(axis=2)).max(axis=1)
    return centre, radius


def ball_slack(K: np.ndarray, page: int, centre: np.ndarray, radius: np.ndarray) -> np.ndarray:
    """radius - (largest distance of a key of the page from `centre`), [Hkv, P]: any centre / radius pair
    with no negative entry here encloses its page (what the bound needs; the centre need not be the mean)."""
    K = np.asarray(K, dtype=np.float64)
    Hkv, N, d = K.shape
    out = np.empty(radius.shape)
    for p in range(radius.shape[1]):
        rows = K[:, p * page:min(N, (p + 1) * page)]
        out[:, p] = radius[:, p] - np.sqrt(((rows - centre[:, p][:, None, :]) ** 2).sum(axis=2)).max(axis=1)
    return out


def page_upper_bound(q: np.ndarray, centre: np.ndarray, radius: np.ndarray, beta: float = 1.0) -> np.ndarray:
    """q [Hq, d], balls of [Hkv, P] pages -> bound [Hq, P] for query head h against the pages of KV head
    h // G: the centre's score plus beta |q| r."""
    q = np.asarray(q, dtype=np.float64)
    Hq, d = q.shape
    G = Hq // centre.shape[0]
    out = np.empty((Hq, centre.shape[1]))
    for h in range(Hq):
        out[h] = centre[h // G] @ q[h] + beta * np.sqrt(q[h] @ q[h]) * radius[h // G]
    return out


def pages_holding_topk(idx: np.ndarray, n_pages: int, page: int, G: int) -> np.ndarray:
    """idx [Hq, k] selected positions (-1 padded) -> bool [Hkv, P]: pages of a KV head that hold at
    least one selected key of one of its query heads (what any exact search has to read)."""
    Hq = idx.shape[0]
    need = np.zeros((Hq // G, n_pages), dtype=bool)
    for h in range(Hq):
        sel = idx[h][idx[h] >= 0]
        need[h // G, np.unique(sel // page)] = True
    return need


def pages_above(bound: np.ndarray, level: np.ndarray, G: int) -> np.ndarray:
    """bound [Hq, P], level [Hq] -> bool [Hkv, P]: pages whose bound reaches the level of at least one
    query head of the KV head (the pages a search with per-head cut-offs `level` reads)."""
    Hq, P = bound.shape
    keep = bound >= np.asarray(level, dtype=np.float64)[:, None]
    return keep.reshape(Hq // G, G, P).any(axis=1)


def search_in_pages(S: np.ndarray, keep: np.ndarray, k: int, page: int, G: int):
    """The search restricted to the pages read: S [Hq, N] scores, keep [Hkv, P] -> list of index
    arrays (descending score, ties to the lower position), the k best keys among the pages kept."""
    Hq, N = S.shape
    out = []
    for h in range(Hq):
        pos = np.nonzero(np.repeat(keep[h // G], page)[:N])[0]
        order = pos[np.lexsort((pos, -S[h, pos]))]
        out.append(order[:k])
    return out
