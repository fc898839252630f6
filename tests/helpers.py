"""Shared test helpers: margin enforcement (uses the oracle), upload, parity checks."""
from __future__ import annotations

import numpy as np

from oracle import c_oracle
from oracle import topk_attention_ref as ref_np
from paper_2502_06766_amd import workloads as wl

U32 = 2.0 ** -24   # unit roundoff of fp32


def abs_storage(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == wl.BF16:
        return x & np.uint16(0x7FFF)
    return np.abs(x)


def scale_rows_storage(K: np.ndarray, dtype: int, g: int, rows: np.ndarray, factor: float) -> None:
    """K[g, rows] *= factor, re-rounded to the storage dtype (in place)."""
    if dtype == wl.BF16:
        f = wl.bf16_bits_to_f32(K[g, rows]) * np.float32(factor)
        K[g, rows] = wl.to_bf16_bits(f)
    else:
        K[g, rows] = (K[g, rows].astype(np.float32) * np.float32(factor)).astype(K.dtype)


def score_margin(q, K, dtype) -> np.ndarray:
    """delta_h = 8 d u max_i sum_c |q_c K_ic|: four times the worst-case gap two fp32
    dot products of length d can be off by (each is within d u sum|q_c K_ic| of exact)."""
    d = q.shape[1]
    A = c_oracle.scores(abs_storage(q, dtype), abs_storage(K, dtype), dtype)
    return 8.0 * d * U32 * A.max(axis=1)


def enforce_margin(q, K, dtype, k, max_rounds=60, prefix=None, shrink=2.0 ** -6):
    """Nudge keys (scale the row by 1 - shrink) until, for every head and every k asked
    for (an int or a list), no unselected score lies within delta_h below the k-th largest
    score.  `prefix[h]` (default N) is the number of leading keys head h searches.  Uses only
    oracle scores.  Returns (K, delta [Hq], rounds).  K is modified in place.

    A nudged key moves in every head that shares its KV head; when it drops out of another
    head's selection that head's boundary moves to a score whose neighbourhood has not been
    cleared yet.  With many rows per KV head and a large N use a smaller `shrink` (still
    several ulps of the storage dtype) so that such crossings stay rare and the rounds converge."""
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    P = np.full(Hq, N, dtype=np.int64) if prefix is None else np.asarray(prefix, dtype=np.int64)
    ks = list(k) if isinstance(k, (list, tuple)) else [k]
    delta = score_margin(q, K, dtype)
    if all(kk >= P.max() for kk in ks):
        return K, delta, 0
    for rnd in range(max_rounds):
        S = c_oracle.scores(q, K, dtype)
        dirty = False
        for h in range(Hq):
            n = int(P[h])
            s = S[h, :n]
            for kk in ks:
                if kk >= n:
                    continue
                part = np.partition(s, n - kk)          # part[n-kk] is the kk-th largest
                s_k = part[n - kk]
                below = part[:n - kk]
                if below.max() > s_k - delta[h]:
                    # unselected keys inside the band (ties with s_k at higher positions included)
                    cand = np.nonzero(s > s_k - delta[h])[0]      # the kk selected plus the band
                    order = cand[np.lexsort((cand, -s[cand]))]
                    viol = order[kk:]
                    scale_rows_storage(K, dtype, h // G, viol, 1.0 - shrink)
                    dirty = True
                    break    # scores of this KV head changed: re-score before looking further
        if not dirty:
            return K, delta, rnd
    raise MarginNotReached("margin enforcement did not converge")


def rows_by_kv_head(q, Hkv):
    """q [M, Hq, d] -> [Hkv * M * G, d] with all (query, head) rows of a KV head adjacent
    (row kvh * M * G + m * G + g is head kvh * G + g of query m), so that the single-query
    helpers apply with a head group of M * G."""
    M, Hq, d = q.shape
    G = Hq // Hkv
    return np.ascontiguousarray(q.reshape(M, Hkv, G, d).transpose(1, 0, 2, 3).reshape(Hkv * M * G, d))


def multi_prefix(M, Hq, Hkv, N, causal, window):
    """Searched prefix length of every row of rows_by_kv_head."""
    G = Hq // Hkv
    P = np.empty((Hkv, M, G), dtype=np.int64)
    for m in range(M):
        n_vis = N - (M - 1 - m) if causal else N
        P[:, m, :] = n_vis - min(window, n_vis)
    return P.reshape(-1)


def enforce_margin_multi(q, K, dtype, k, causal, window=0, shrink=2.0 ** -6):
    """Margin enforcement for a chunk of queries q [M, Hq, d]; returns (K, delta [M, Hq])."""
    M, Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    q2 = rows_by_kv_head(q, Hkv)
    K, delta2, _ = enforce_margin(q2, K, dtype, k, prefix=multi_prefix(M, Hq, Hkv, N, causal, window), shrink=shrink)
    delta = delta2.reshape(Hkv, M, G).transpose(1, 0, 2).reshape(M, Hq)
    return K, delta


def to_torch(x: np.ndarray, dtype: int, device):
    import torch
    if dtype == wl.BF16:
        return torch.from_numpy(x.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(x).to(device)


def check_against_oracle(out, idx, vals, lse, ref, delta, k_eff, tol, vmax, label=""):
    """out/idx/vals/lse: numpy arrays from the GPU for one sequence ([Hq, ...]);
    ref = (out, idx, vals, lse) from the oracle."""
    r_out, r_idx, r_vals, r_lse = ref
    Hq = r_out.shape[0]
    for h in range(Hq):
        got = np.sort(idx[h, :k_eff].astype(np.int64))
        want = np.sort(r_idx[h, :k_eff])
        if not np.array_equal(got, want):
            miss = np.setdiff1d(want, got).size
            raise AssertionError(f"{label} head {h}: index set differs ({miss} of {k_eff} missing)")
        if idx.shape[1] > k_eff:
            assert (idx[h, k_eff:] == -1).all(), f"{label} head {h}: idx padding"
            assert np.isneginf(vals[h, k_eff:]).all(), f"{label} head {h}: vals padding"
        if k_eff > 0:
            gv = np.sort(vals[h, :k_eff].astype(np.float64))[::-1]
            dv = np.abs(gv - r_vals[h, :k_eff]).max()
            assert dv <= delta[h] / 8 + 1e-30, f"{label} head {h}: vals off by {dv} (allowed {delta[h] / 8})"
            # vals must belong to the indices they are reported with
            o = np.argsort(idx[h, :k_eff], kind="stable")
            ro = np.argsort(r_idx[h, :k_eff], kind="stable")
            dv2 = np.abs(vals[h, :k_eff][o].astype(np.float64) - r_vals[h, :k_eff][ro]).max()
            assert dv2 <= delta[h] / 8 + 1e-30, f"{label} head {h}: vals not aligned with idx ({dv2})"
        scale = max(np.abs(r_out[h]).max(), 1e-6 * vmax)
        err = np.abs(out[h].astype(np.float64) - r_out[h]).max() / scale
        assert err <= tol, f"{label} head {h}: out rel err {err:.3e} > {tol}"
        if lse is not None:
            assert abs(lse[h] - r_lse[h]) <= 1e-4 * max(1.0, abs(r_lse[h])), \
                f"{label} head {h}: lse {lse[h]} vs {r_lse[h]}"


def out_tolerance(dtype: int) -> float:
    """2e-3 relative for 16-bit K/V with fp32 accumulate, 1e-5 for fp32."""
    return 1e-5 if dtype == wl.F32 else 2e-3


class MarginNotReached(AssertionError):
    """enforce_margin ran out of rounds (dense k with many rows per KV head): the case is judged by
    check_unmargined instead, which needs no margin."""


def check_unmargined(res, q, K, V, dtype, k, window=0, label="", S=None):
    """Judges one query's result on inputs WITHOUT an enforced margin, against the oracle alone.
    res = (out, idx, vals, lse) numpy arrays [Hq, ...] (vals / lse may be None); q [Hq, d]; K, V [Hkv, N, d]
    hold exactly the tokens the query sees.  fp32 and float64 scores may order keys within delta_h of the
    k-th score differently, so:
      * idx must be k_eff distinct positions of the searched prefix, and may differ from the oracle's set
        only among keys whose oracle score lies within delta_h of the k-th oracle score;
      * vals must be the oracle scores at idx (within delta_h / 8);
      * out / lse must equal the oracle's softmax-weighted sum over the positions the GPU selected plus
        the window (the usual tolerance): with an equally valid but different set the oracle's own out
        is not the reference.
    Returns the fraction of heads whose set equals the oracle's exactly."""
    out, idx, vals, lse = res
    Hq, d = q.shape
    Hkv, N, _ = K.shape
    G = Hq // Hkv
    W = min(window, N)
    P = N - W
    k_eff = min(k, P)
    if S is None:
        S = c_oracle.scores(q, K, dtype)
    r_idx = c_oracle.topk_attention_window(q, K, V, dtype, k, window)[1]
    delta = score_margin(q, K, dtype)
    Vw = wl.widen(V, dtype)
    tol = out_tolerance(dtype)
    vmax = float(np.abs(Vw).max())
    same = 0
    for h in range(Hq):
        got = idx[h, :k_eff].astype(np.int64)
        assert (idx[h, k_eff:] == -1).all(), f"{label} head {h}: idx padding"
        if vals is not None:
            assert np.isneginf(vals[h, k_eff:]).all(), f"{label} head {h}: vals padding"
        if k_eff > 0:
            assert np.unique(got).size == k_eff and got.min() >= 0 and got.max() < P, f"{label} head {h}: invalid index"
            want = r_idx[h, :k_eff]
            s_k = np.partition(S[h, :P], P - k_eff)[P - k_eff]
            extra, missing = np.setdiff1d(got, want), np.setdiff1d(want, got)
            same += extra.size == 0
            assert (S[h, extra] >= s_k - delta[h]).all(), f"{label} head {h}: a selected key lies below the band"
            assert (S[h, missing] <= s_k + delta[h]).all(), f"{label} head {h}: a key above the band is missing"
            if vals is not None:
                dv = np.abs(vals[h, :k_eff].astype(np.float64) - S[h, got]).max()
                assert dv <= delta[h] / 8 + 1e-30, f"{label} head {h}: vals off by {dv}"
        else:
            same += 1
        rows = np.concatenate([got, np.arange(P, N)])
        o, l = ref_np.attend_selected(S[h, rows], Vw[h // G][rows], d)
        scale = max(np.abs(o).max(), 1e-6 * vmax)
        err = np.abs(out[h].astype(np.float64) - o).max() / scale
        assert err <= tol, f"{label} head {h}: out rel err {err:.3e} > {tol}"
        if lse is not None:
            assert abs(lse[h] - l) <= 1e-4 * max(1.0, abs(l)), f"{label} head {h}: lse {lse[h]} vs {l}"
    return same / Hq


def check_band_tolerant(out, idx, ref, S, delta, k_eff, tol, vmax, label=""):
    """For inputs WITHOUT an enforced margin: fp32 and float64 scores may order keys that lie within
    delta_h of the k-th score differently, so the index sets may differ, but only there.  S [Hq, N] are
    the oracle's scores.  Returns the fraction of heads whose set equals the oracle's exactly."""
    r_out, r_idx = ref[0], ref[1]
    Hq = r_out.shape[0]
    same = 0
    for h in range(Hq):
        got = np.unique(idx[h, :k_eff].astype(np.int64))
        assert got.size == k_eff and got.min() >= 0 and got.max() < S.shape[1], f"{label} head {h}: invalid index"
        want = np.sort(r_idx[h, :k_eff])
        s_k = np.sort(S[h])[::-1][k_eff - 1]
        extra, missing = np.setdiff1d(got, want), np.setdiff1d(want, got)
        same += extra.size == 0
        assert (S[h, extra] >= s_k - delta[h]).all(), f"{label} head {h}: a selected key lies below the band"
        assert (S[h, missing] <= s_k + delta[h]).all(), f"{label} head {h}: a key above the band is missing"
        scale = max(np.abs(r_out[h]).max(), 1e-6 * vmax)
        err = np.abs(out[h].astype(np.float64) - r_out[h]).max() / scale
        assert err <= tol, f"{label} head {h}: out rel err {err:.3e} > {tol}"
    return same / Hq
