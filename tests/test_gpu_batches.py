"""GPU tests of batched use: the per-step append for a whole batch (Algorithm 1's concat for every
sequence of a layer in one call) must leave the cache bytes, the int8 index and the lengths that
per-sequence appends leave, and decodes over batches of many sequences (short ones on the general
path, long ones on the filtered path) must match the oracle."""
import numpy as np
import pytest
import torch

import helpers as H
from oracle import c_oracle
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None


@pytest.mark.parametrize("dtype,d,index", [(wl.F16, 128, True), (wl.BF16, 64, True), (wl.F32, 64, False),
                                           (wl.F16, 32, False), (wl.BF16, 256, True)])
def test_append_step_equals_per_sequence_appends(dtype, d, index):
    g = np.random.default_rng(1000 + d + dtype)
    L, B, Hq, Hkv, Ncap = 2, 3, 8, 2, 900
    start = [300, 0, 517]                       # ragged lengths before the batched steps
    steps = [1, 1, 3, 1, 17, 150, 1]            # tokens per batched append (one workgroup's worth, or many)
    total = [s + sum(steps) for s in start]
    k = 40
    q = wl.quantize(g.standard_normal((B, Hq, d)).astype(np.float32), dtype)
    K = wl.quantize(g.standard_normal((B, Hkv, max(total), d)).astype(np.float32), dtype)
    V = wl.quantize(g.standard_normal((B, Hkv, max(total), d)).astype(np.float32), dtype)
    for s in range(B):                          # a score margin at the k-th boundary of what the decode will see
        Ks, _, _ = H.enforce_margin(q[s], np.ascontiguousarray(K[s, :, :total[s]]), dtype, k)
        K[s, :, :total[s]] = Ks
    Kd, Vd = H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV)
    kind = ta.INDEX_INT8 if index else ta.INDEX_NONE
    a = ta.TopkAttnCache(L, B, Hq, Hkv, d, Ncap, 64, dtype, index_kind=kind)
    b = ta.TopkAttnCache(L, B, Hq, Hkv, d, Ncap, 64, dtype, index_kind=kind)
    try:
        a.kv.zero_(); b.kv.zero_()
        layer = 1
        for s in range(B):
            if start[s]:
                for c in (a, b):
                    c.append(layer, s, Kd[s, :, :start[s]].contiguous(), Vd[s, :, :start[s]].contiguous(),
                             head_major=True)
        pos = list(start)
        for n in steps:
            kn = torch.stack([Kd[s, :, pos[s]:pos[s] + n].permute(1, 0, 2) for s in range(B)]).contiguous()
            vn = torch.stack([Vd[s, :, pos[s]:pos[s] + n].permute(1, 0, 2) for s in range(B)]).contiguous()
            a.append_step(layer, kn, vn)                       # [B, n, Hkv, d]
            for s in range(B):
                b.append(layer, s, kn[s], vn[s])
                pos[s] += n
        torch.cuda.synchronize()
        assert [a.length(layer, s) for s in range(B)] == total
        assert [a.length(0, s) for s in range(B)] == [0] * B
        assert torch.equal(a.kv, b.kv)                         # keys, values, codes and scales, byte for byte
        # the device-side lengths moved too: a decode sees every appended token
        out, idx, vals, lse = a.decode(layer, H.to_torch(q, dtype, DEV), k)
        torch.cuda.synchronize()
        for s in range(B):
            Ks, Vs = np.ascontiguousarray(K[s, :, :total[s]]), np.ascontiguousarray(V[s, :, :total[s]])
            ref = c_oracle.topk_attention(q[s], Ks, Vs, dtype, k)
            H.check_against_oracle(out[s].cpu().numpy(), idx[s].cpu().numpy(), vals[s].cpu().numpy(),
                                   lse[s].cpu().numpy(), ref, H.score_margin(q[s], Ks, dtype), min(k, total[s]),
                                   H.out_tolerance(dtype), float(np.abs(wl.widen(Vs, dtype)).max()), f"seq {s}")
    finally:
        a.close(); b.close()


def test_append_step_capacity_and_arguments():
    d, B = 64, 2
    c = ta.TopkAttnCache(1, B, 4, 2, d, 300, 16, wl.F16)
    try:
        kn = torch.zeros(B, 8, 2, d, dtype=torch.float16, device=DEV)
        c.append(0, 1, kn[0, :8].repeat(37, 1, 1)[:290].contiguous(), kn[0, :8].repeat(37, 1, 1)[:290].contiguous())
        c.append_step(0, kn, kn)                                # 298 <= 300 for the longer sequence
        assert [c.length(0, s) for s in range(B)] == [8, 298]
        with pytest.raises(ta.TopkAttnError) as e:
            c.append_step(0, kn, kn)                            # 306 > 300: nothing is appended anywhere
        assert e.value.code == ta.ECAPACITY
        assert [c.length(0, s) for s in range(B)] == [8, 298]
        assert ta.lib().topk_attn_append_step(c.h, 0, None, None, 0, None) == ta.OK       # n_new = 0: no-op
        assert ta.lib().topk_attn_append_step(c.h, 0, None, None, 1, None) == ta.EINVAL
        assert ta.lib().topk_attn_append_step(c.h, 1, kn.data_ptr(), kn.data_ptr(), 1, None) == ta.EINVAL
    finally:
        c.close()


def test_serving_batch_of_many_short_sequences():
    """1500 sequences of 1..400 tokens in one call, grown by batched appends: the grid dimensions
    that carry the sequence index, ragged lengths inside one launch, k above and below the lengths."""
    dtype, Hq, Hkv, d, k, B = wl.F16, 8, 2, 64, 24, 1500
    g = np.random.default_rng(77)
    lens = g.integers(1, 401, size=B)
    lens[:4] = [1, 400, 24, 25]
    Nmax = int(lens.max())
    K = wl.quantize(g.standard_normal((B, Hkv, Nmax, d)).astype(np.float32), dtype)
    V = wl.quantize(g.standard_normal((B, Hkv, Nmax, d)).astype(np.float32), dtype)
    q = wl.quantize(g.standard_normal((B, Hq, d)).astype(np.float32), dtype)
    check = list(range(8)) + g.choice(B, size=40, replace=False).tolist() + [B - 1]
    for s in check:                                     # a score margin where the result is compared
        n = int(lens[s])
        K[s, :, :n] = H.enforce_margin(q[s], np.ascontiguousarray(K[s, :, :n]), dtype, k)[0]
    cache = ta.TopkAttnCache(1, B, Hq, Hkv, d, Nmax + 2, k, dtype)
    try:
        Kd, Vd = H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV)
        # every sequence starts with its first token, then batched steps add a token to all of them;
        # sequences that are already complete receive a copy of their last token, removed again below
        # by resetting and re-importing them
        for s in range(B):
            n = int(lens[s])
            cache.append(0, s, Kd[s, :, :max(1, n - 2)].contiguous(), Vd[s, :, :max(1, n - 2)].contiguous(),
                         head_major=True)
        for step in range(2):
            pos = torch.tensor(np.clip(np.maximum(1, lens - 2) + step, 0, Nmax - 1), device=DEV)
            kn = Kd[torch.arange(B, device=DEV), :, pos][:, None].contiguous()     # [B, 1, Hkv, d]
            vn = Vd[torch.arange(B, device=DEV), :, pos][:, None].contiguous()
            cache.append_step(0, kn, vn)
        short = [s for s in range(B) if lens[s] < 3]    # these got more tokens than they have
        for s in short:
            cache.reset(0, s)
            n = int(lens[s])
            cache.append(0, s, Kd[s, :, :n].contiguous(), Vd[s, :, :n].contiguous(), head_major=True)
        assert [cache.length(0, s) for s in range(B)] == lens.tolist()
        out, idx, vals, lse = cache.decode(0, H.to_torch(q, dtype, DEV), k)
        torch.cuda.synchronize()
        out, idx, vals, lse = (t.cpu().numpy() for t in (out, idx, vals, lse))
        for s in check:
            n = int(lens[s])
            Ks, Vs = np.ascontiguousarray(K[s, :, :n]), np.ascontiguousarray(V[s, :, :n])
            ref = c_oracle.topk_attention(q[s], Ks, Vs, dtype, k)
            H.check_against_oracle(out[s], idx[s], vals[s], lse[s], ref, H.score_margin(q[s], Ks, dtype), min(k, n),
                                   H.out_tolerance(dtype), float(np.abs(wl.widen(Vs, dtype)).max()), f"seq {s}")
        # the sequences not compared one by one: valid positions, no duplicates, padding where k > length
        for s in range(B):
            n, ke = int(lens[s]), min(k, int(lens[s]))
            for h in range(Hq):
                sel = idx[s, h, :ke]
                assert sel.min() >= 0 and sel.max() < n and np.unique(sel).size == ke, f"seq {s} head {h}"
                assert (idx[s, h, ke:] == -1).all()
            assert np.isfinite(out[s]).all()
    finally:
        cache.close()


def test_batch_of_40_sequences_on_the_filtered_path():
    """1280 heads in one call, ragged lengths of 33k..41k tokens: the filtered scan with the small
    workgroups the threshold and candidate selections take when a call has many heads."""
    dtype, Hq, Hkv, d, k, B = wl.BF16, 32, 8, 64, 300, 40
    g = np.random.default_rng(5)
    lens = g.integers(33000, 41000, size=B)
    Nmax = int(lens.max())
    q = wl.quantize(g.standard_normal((B, Hq, d)).astype(np.float32), dtype)
    base_K = wl.quantize(g.standard_normal((Hkv, Nmax + 4096, d)).astype(np.float32), dtype)
    base_V = wl.quantize(g.standard_normal((Hkv, Nmax + 4096, d)).astype(np.float32), dtype)
    cache = ta.TopkAttnCache(1, B, Hq, Hkv, d, Nmax, k, dtype)
    try:
        host = []
        for s in range(B):                          # every sequence: its own window of the base arrays
            n, o = int(lens[s]), 97 * s
            Ks = np.ascontiguousarray(base_K[:, o:o + n])
            Ks = H.enforce_margin(q[s], Ks, dtype, k)[0]
            Vs = np.ascontiguousarray(base_V[:, o:o + n])
            host.append((Ks, Vs))
            cache.append(0, s, H.to_torch(Ks, dtype, DEV), H.to_torch(Vs, dtype, DEV), head_major=True)
        out, idx, vals, lse = cache.decode(0, H.to_torch(q, dtype, DEV), k)
        torch.cuda.synchronize()
        assert cache.last_fallbacks() == 0
        out, idx, vals, lse = (t.cpu().numpy() for t in (out, idx, vals, lse))
        for s in range(B):
            Ks, Vs = host[s]
            ref = c_oracle.topk_attention(q[s], Ks, Vs, dtype, k)
            H.check_against_oracle(out[s], idx[s], vals[s], lse[s], ref, H.score_margin(q[s], Ks, dtype), k,
                                   H.out_tolerance(dtype), float(np.abs(wl.widen(Vs, dtype)).max()), f"seq {s}")
    finally:
        cache.close()
