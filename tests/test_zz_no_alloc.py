"""topk_attn_decode_static (the entry point that allocates nothing: its per-call buffers live in
an array built into the library) against topk_attn_decode on the same handle, through the C ABI.
Same kernels in the same order, so the bar is the strictest one: bit-identical out / idx / vals /
lse.  Two calls in a row, the second on a smaller input, then the size limit."""
import ctypes

import numpy as np
import pytest
import torch

import helpers as H
from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = torch.device("cuda", 0) if torch.cuda.is_available() else None


def _decode_both(cache, layer, qd, k, Hq, d):
    """(reference through topk_attn_decode, result through topk_attn_decode_static)."""
    L = ta.lib()
    st = torch.cuda.current_stream().cuda_stream
    res = []
    for fn in (L.topk_attn_decode, L.topk_attn_decode_static):
        out = torch.full((1, Hq, d), float("nan"), dtype=torch.float32, device=DEV)
        idx = torch.full((1, Hq, k), -7, dtype=torch.int32, device=DEV)
        vals = torch.full((1, Hq, k), float("nan"), dtype=torch.float32, device=DEV)
        lse = torch.full((1, Hq), float("nan"), dtype=torch.float32, device=DEV)
        rc = fn(cache.h, layer, qd.data_ptr(), k, out.data_ptr(), idx.data_ptr(), vals.data_ptr(), lse.data_ptr(), st)
        assert rc == ta.OK, ta.topk_attn_strerror(rc)
        torch.cuda.synchronize()
        res.append((out, idx, vals, lse, cache.last_fallbacks()))
    return res


def test_static_scratch_decode_matches_decode_twice_then_smaller():
    dtype, Hq, Hkv, d = wl.F16, 8, 2, 128
    g = np.random.default_rng(4242)
    # layer 0: 50001 tokens, k = 700 (filtered scan); layer 1: 3000 tokens, k = 40 (general path);
    # a second handle with all keys identical: every head's candidate list overflows and is redone exactly
    cases = [(0, 50001, 700), (1, 3000, 40)]
    cache = ta.TopkAttnCache(2, 1, Hq, Hkv, d, 50001, 700, dtype)
    try:
        qs = {}
        for layer, n, k in cases:
            q = wl.quantize(g.standard_normal((Hq, d)).astype(np.float32), dtype)
            K = wl.quantize(g.standard_normal((Hkv, n, d)).astype(np.float32), dtype)
            V = wl.quantize(g.standard_normal((Hkv, n, d)).astype(np.float32), dtype)
            cache.append(layer, 0, H.to_torch(K, dtype, DEV), H.to_torch(V, dtype, DEV), head_major=True)
            qs[layer] = H.to_torch(q, dtype, DEV)[None].contiguous()
        for layer, n, k in cases + [cases[0]]:      # large, smaller, large again
            print(f"static decode: layer {layer} N={n} k={k}", flush=True)
            ref, got = _decode_both(cache, layer, qs[layer], k, Hq, d)
            for a, b, name in zip(ref[:4], got[:4], ("out", "idx", "vals", "lse")):
                assert torch.equal(a, b), f"layer {layer}: {name} differs between decode and decode_static"
            assert ref[4] == got[4] == 0
            assert not torch.isnan(got[0]).any() and (got[1] >= 0).all()
        # without idx / vals / lse outputs the selection lands in the built-in buffer too
        out = torch.empty((1, Hq, d), dtype=torch.float32, device=DEV)
        rc = ta.lib().topk_attn_decode_static(cache.h, 0, qs[0].data_ptr(), 700, out.data_ptr(), None, None, None,
                                              torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert rc == ta.OK and torch.equal(out, _decode_both(cache, 0, qs[0], 700, Hq, d)[0][0])
    finally:
        cache.close()

    # exact redo of every head (its score rows live in the built-in buffer as well), on a smaller cache
    N, k = 150000, 77
    q = wl.quantize(g.integers(-2, 3, (4, d)).astype(np.float32), wl.BF16)
    K = np.tile(wl.quantize(g.integers(-2, 3, (1, 1, d)).astype(np.float32), wl.BF16), (1, N, 1))
    V = wl.quantize(g.standard_normal((1, N, d)).astype(np.float32), wl.BF16)
    cache = ta.TopkAttnCache(1, 1, 4, 1, d, N, k, wl.BF16)
    try:
        cache.set_path(ta.PATH_FILTER)
        cache.append(0, 0, H.to_torch(K, wl.BF16, DEV), H.to_torch(V, wl.BF16, DEV), head_major=True)
        print("static decode: identical keys, every head redone", flush=True)
        ref, got = _decode_both(cache, 0, H.to_torch(q, wl.BF16, DEV)[None].contiguous(), k, 4, d)
        for a, b in zip(ref[:4], got[:4]):
            assert torch.equal(a, b)
        assert ref[4] == got[4] == 4
        assert torch.equal(torch.sort(got[1][0], dim=1).values,
                           torch.arange(k, dtype=torch.int32, device=DEV).expand(4, k))
    finally:
        cache.close()


def test_static_scratch_rejects_what_does_not_fit():
    """One million-token layer needs 128 MiB of score rows alone: ESCRATCH, nothing enqueued."""
    d, N, k = 128, 1 << 20, 16384
    cfg = ta.make_config(1, 1, 32, 8, d, N, k, ta.F16)
    assert ta.topk_attn_workspace_bytes(cfg) > (96 << 20)
    cache = ta.TopkAttnCache(1, 1, 32, 8, d, N, k, ta.F16)
    try:
        kv = torch.zeros((8, 64, d), dtype=torch.float16, device=DEV)
        cache.append(0, 0, kv, kv, head_major=True)
        q = torch.zeros((1, 32, d), dtype=torch.float16, device=DEV)
        out = torch.full((1, 32, d), 5.0, dtype=torch.float32, device=DEV)
        rc = ta.lib().topk_attn_decode_static(cache.h, 0, q.data_ptr(), 8, out.data_ptr(), None, None, None, None)
        assert rc == ta.ESCRATCH and "scratch" in ta.topk_attn_strerror(rc)
        torch.cuda.synchronize()
        assert (out == 5.0).all()
        assert ta.lib().topk_attn_decode(cache.h, 0, q.data_ptr(), 8, out.data_ptr(), None, None, None, None) == ta.OK
        torch.cuda.synchronize()
    finally:
        cache.close()
    assert ta.lib().topk_attn_decode_static(None, 0, None, 1, None, None, None, None, None) == ta.EINVAL
