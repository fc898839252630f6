"""CPU oracle for the compressed (int8) key index.  TEST INFRASTRUCTURE.

The paper's search index may be a plain list (exact search) or an approximate structure
(methodology section, the paragraph on converting the key tensors into a search index).  The index checked here is the usual compressed-list kind of vector
databases: every key row is stored a second time as int8 codes with one fp32 scale per
row, the query is coded the same way, approximate scores come from the integer dot
product, and a candidate set chosen by approximate score is re-scored exactly before the
final top-k (approximate search, exact refinement).  The paper fixes none of these
details; the definitions below are this build's and are listed with its other readings.

  code_c  = rint(x_c * (127 / amax))    (fp32 multiply, round half to even), amax = max_c |x_c|
  scale   = amax / 127                  (fp32); a row with amax < 2^-100 (all zeros included) has
                                        codes 0 and scale 0, which keeps 127 / amax finite
  s~(q,K_i) = float(sum_c codeq_c * codeK_ic) * (scale_q * scale_Ki)     (all fp32)

Encoding and integer work are bit-exact contracts; the search result is judged by
recall@k against the exact oracle (topk_attention_ref) and by the output tolerance.
Only tests may import this file; it shares no code with the HIP path.

Pins (tests/test_oracle_pins.py): reconstruction error <= scale / 2 per element, the
largest element maps to +-127, sign symmetry, monotonicity, agreement with the library
quantiser (torch.quantize_per_tensor) up to its own rounding of 1/scale, the closed-form
bound on |s~ - s|, rerank with all N candidates equals the exact step, recall is
non-decreasing in the candidate count.  No function is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from oracle import topk_attention_ref as ref


def quantize_rows_int8(x: np.ndarray):
    """x [..., d] (values exactly representable in fp32) -> (codes int8 [..., d], scale fp32 [...])."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.abs(x).max(axis=-1)
    live = amax >= np.float32(2.0 ** -100)
    safe = np.where(live, amax, np.float32(1.0))
    inv = np.where(live, np.float32(127.0) / safe, np.float32(0.0)).astype(np.float32)
    v = (x * inv[..., None]).astype(np.float32)
    codes = np.rint(v).astype(np.int8)               # round half to even, |v| <= 127
    scale = np.where(live, amax / np.float32(127.0), np.float32(0.0)).astype(np.float32)
    return codes, scale


def approx_scores_int8(q: np.ndarray, K: np.ndarray) -> np.ndarray:
    """Approximate score matrix [Hq, N] (fp32) from the coded query and keys.
    q [Hq, d], K [Hkv, N, d]; query head h reads KV head h // G."""
    cq, sq = quantize_rows_int8(q)
    cK, sK = quantize_rows_int8(K)
    Hq = q.shape[0]
    G = Hq // K.shape[0]
    out = np.empty((Hq, K.shape[1]), dtype=np.float32)
    for h in range(Hq):
        dot = cK[h // G].astype(np.int64) @ cq[h].astype(np.int64)          # exact
        out[h] = dot.astype(np.float32) * (sq[h] * sK[h // G]).astype(np.float32)
    return out


def rerank_topk(q, K, V, k: int, n_candidates: int):
    """Approximate search with exact refinement for one (layer, sequence): per head take the
    n_candidates positions with the largest approximate scores (ties to the lower position),
    score them exactly, keep the k best (exact score, ties to the lower position) and attend
    over them.  Returns (out [Hq, d], idx [Hq, k], vals [Hq, k], lse [Hq]) like the exact step."""
    q64 = np.asarray(q, dtype=np.float64)
    K64 = np.asarray(K, dtype=np.float64)
    V64 = np.asarray(V, dtype=np.float64)
    Hq, d = q64.shape
    Hkv, N, _ = K64.shape
    G = Hq // Hkv
    A = approx_scores_int8(q, K)
    S = ref.scores(q64, K64)
    c = min(int(n_candidates), N)
    out = np.zeros((Hq, d))
    idx = np.full((Hq, k), -1, dtype=np.int64)
    vals = np.full((Hq, k), -np.inf)
    lse = np.zeros(Hq)
    for h in range(Hq):
        cand, _ = ref.select_topk(A[h].astype(np.float64), c)
        cand = np.sort(cand)
        I_local, v = ref.select_topk(S[h, cand], k)         # ties to the lower local = lower global position
        I = cand[I_local]
        idx[h, :I.shape[0]] = I
        vals[h, :I.shape[0]] = v
        out[h], lse[h] = ref.attend_selected(v, V64[h // G][I], d)
    return out, idx, vals, lse


def recall_at_k(idx_got: np.ndarray, idx_ref: np.ndarray) -> float:
    """Share of the reference positions (entries >= 0) that were returned, for one head."""
    want = set(int(i) for i in np.asarray(idx_ref).ravel() if i >= 0)
    got = set(int(i) for i in np.asarray(idx_got).ravel() if i >= 0)
    return 1.0 if not want else len(want & got) / len(want)
