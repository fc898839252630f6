"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, sizes caches as the paper's 2NDL formula says, and rejects
bad configurations before touching a device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2502_06766_amd import topk_attn as ta
from paper_2502_06766_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in ("topk_attn.h", "topk_attn_debug.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(topk_attn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ta.lib()
    names = header_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), f"{n} declared in topk_attn.h but not exported"
    assert sorted(ta.EXPORTS) == names


def test_config_struct_matches_header_size():
    # uint32 + 5*int32 + int64 + 6*int32 + 2*(ptr + size_t) = 24 + 8 + 24 + 32
    assert ctypes.sizeof(ta.Config) == 88


def test_kv_bytes_is_2ndl():
    # Llama-3-8B-like layer shapes with GQA: 2 * L * B * Hkv * Ncap * d * e
    cfg = ta.make_config(32, 1, 32, 8, 128, 524288, 8192, ta.F16)
    assert ta.topk_attn_kv_bytes(cfg) == 2 * 32 * 8 * 524288 * 128 * 2
    # the paper's own example ignores GQA: hidden 4096 = 32 heads of 128, N = 100k, 16 bit
    cfg = ta.make_config(32, 1, 32, 32, 128, 100000, 1000, ta.BF16)
    got = ta.topk_attn_kv_bytes(cfg)
    assert abs(got - wl.kv_cache_bytes(100000, 4096, 32, 2)) <= 2 * 256
    assert abs(got / 1e9 - 52) < 1.0
    assert ta.topk_attn_workspace_bytes(cfg) > 0


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), ta.EUNSUPPORTED),
    (dict(dtype=7), ta.EUNSUPPORTED),
    (dict(n_q_heads=30), ta.EUNSUPPORTED),          # 30 % 8 != 0
    (dict(n_q_heads=8 * 129), ta.EUNSUPPORTED),      # group of 129 > 128
    (dict(n_q_heads=8 * 32, dtype=ta.F32), ta.EUNSUPPORTED),   # fp32 caches: groups up to 16
    (dict(n_layers=0), ta.EINVAL),
    (dict(max_k=0), ta.EINVAL),
    (dict(max_tokens=1 << 31), ta.EINVAL),
    (dict(max_queries=-1), ta.EINVAL),
    (dict(max_queries=5000), ta.EINVAL),
    (dict(n_seqs=4096, max_queries=16), ta.EINVAL),  # sequences x queries is a grid dimension
])
def test_bad_config_rejected_without_device(kw, code):
    base = dict(n_layers=1, n_seqs=1, n_q_heads=32, n_kv_heads=8, head_dim=128, max_tokens=4096, max_k=64,
                dtype=ta.F16)
    base.update(kw)
    cfg = ta.make_config(**base)
    assert ta.topk_attn_kv_bytes(cfg) == 0
    assert ta.topk_attn_workspace_bytes(cfg) == 0
    h = ctypes.c_void_p()
    assert ta.lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)) == code
    assert not h.value


def test_workspace_grows_with_max_queries():
    one = ta.topk_attn_workspace_bytes(ta.make_config(1, 2, 32, 8, 128, 65536, 1024, ta.F16))
    same = ta.topk_attn_workspace_bytes(ta.make_config(1, 2, 32, 8, 128, 65536, 1024, ta.F16, max_queries=1))
    four = ta.topk_attn_workspace_bytes(ta.make_config(1, 2, 32, 8, 128, 65536, 1024, ta.F16, max_queries=4))
    assert same == one
    assert 3.9 * one < four <= 4 * one
    cfg = ta.make_config(1, 1, 4, 2, 64, 128, 8, ta.F32)
    cfg.index_kind = 7
    assert ta.topk_attn_workspace_bytes(cfg) == 0


def test_int8_index_storage_and_supported_shapes():
    base = dict(n_layers=2, n_seqs=3, n_q_heads=8, n_kv_heads=2, head_dim=128, max_tokens=1000, max_k=64)
    plain = ta.topk_attn_kv_bytes(ta.make_config(dtype=ta.F16, **base))
    with_index = ta.topk_attn_kv_bytes(ta.make_config(dtype=ta.F16, index_kind=ta.INDEX_INT8, **base))
    rows = 2 * 3 * 2 * 1000
    up = lambda x: (x + 255) // 256 * 256
    assert plain == 2 * up(rows * 128 * 2)
    assert with_index == plain + up(rows * 128) + up(rows * 4)        # codes, then one fp32 scale per row
    # fp32 caches, head_dim 32 and head groups above 4 have no int8 index
    for kw in (dict(dtype=ta.F32), dict(dtype=ta.F16, head_dim=32), dict(dtype=ta.F16, n_q_heads=16)):
        cfg = ta.make_config(**{**base, **kw, "index_kind": ta.INDEX_INT8})
        assert ta.topk_attn_kv_bytes(cfg) == 0
        h = ctypes.c_void_p()
        assert ta.lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)) == ta.EUNSUPPORTED


def test_create_rejects_null_storage_and_wrong_struct_size():
    cfg = ta.make_config(1, 1, 4, 2, 64, 128, 8, ta.F32)
    h = ctypes.c_void_p()
    assert ta.lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)) == ta.EINVAL   # null storage
    cfg.struct_size = 12
    assert ta.lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)) == ta.EINVAL
    assert ta.lib().topk_attn_create(ctypes.byref(cfg), None) == ta.EINVAL


def test_null_handle_calls_fail_cleanly():
    L = ta.lib()
    assert L.topk_attn_decode(None, 0, None, 1, None, None, None, None, None) == ta.EINVAL
    assert L.topk_attn_decode_multi(None, 0, None, 2, 1, 1, 0, None, None, None, None, None) == ta.EINVAL
    assert L.topk_attn_append_kv(None, 0, 0, None, None, 1, 1, 1, None) == ta.EINVAL
    assert L.topk_attn_length(None, 0, 0) == -1
    assert L.topk_attn_destroy(None) == ta.EINVAL
    assert L.topk_attn_set_path(None, 0) == ta.EINVAL
    assert L.topk_attn_read_probe(None, 16, None, None) == ta.EINVAL


def test_strerror():
    assert ta.topk_attn_strerror(ta.OK) == "ok"
    assert "capacity" in ta.topk_attn_strerror(ta.ECAPACITY)
    assert ta.topk_attn_strerror(99) == "unknown error"


# ---------------------------------------------------------------- layer-wise k schedule (host only)
def test_k_schedule_closed_forms_and_invariants():
    from oracle import topk_attention_ref as ref
    # uniform: equal shares, remainder spread one each
    assert ta.topk_attn_k_schedule(32 * 8192, 32, 1.0) == [8192] * 32
    ks = ta.topk_attn_k_schedule(100, 8, 1.0)
    assert sum(ks) == 100 and max(ks) - min(ks) == 1
    # two layers, ratio 3: shares 1/4 and 3/4
    assert ta.topk_attn_k_schedule(4000, 2, 3.0) == [1000, 3000]
    # arithmetic progression when it divides: L = 5, ratio 3 -> weights 1, 1.5, 2, 2.5, 3 (sum 10)
    assert ta.topk_attn_k_schedule(1000, 5, 3.0) == [100, 150, 200, 250, 300]
    # ties in the fractional parts go to the later layer (the oracle's own pins fix these values)
    assert ta.topk_attn_k_schedule(10, 4, 1.0) == [2, 2, 3, 3] == ref.k_schedule(10, 4, 1.0)
    assert ta.topk_attn_k_schedule(6, 2, 3.0) == [1, 5] == ref.k_schedule(6, 2, 3.0)
    assert ta.topk_attn_k_schedule(100, 8, 1.0) == ref.k_schedule(100, 8, 1.0)
    for total, L, r in [(262144, 32, 4.0), (1000, 7, 2.5), (33, 32, 8.0), (5000, 3, 0.5), (77, 1, 9.0),
                        (7, 3, 3.0), (11, 3, 2.0), (9, 3, 0.5), (12345, 17, 1.0), (999, 10, 10.0)]:
        ks = ta.topk_attn_k_schedule(total, L, r)
        assert sum(ks) == total and min(ks) >= 1 and len(ks) == L
        assert ks == ref.k_schedule(total, L, r)
        d = np.diff(ks)
        if total >= 8 * L:      # linear up to rounding: second differences within +-2
            assert (np.abs(np.diff(d)) <= 2).all()
            assert (d >= -1).all() if r >= 1 else (d <= 1).all()


def test_k_schedule_rejects_bad_arguments():
    buf = (ctypes.c_int32 * 4)()
    L = ta.lib()
    assert L.topk_attn_k_schedule(3, 4, 1.0, buf) == ta.EINVAL          # fewer keys than layers
    assert L.topk_attn_k_schedule(100, 0, 1.0, buf) == ta.EINVAL
    assert L.topk_attn_k_schedule(100, 4, 0.0, buf) == ta.EINVAL
    assert L.topk_attn_k_schedule(100, 4, float("nan"), buf) == ta.EINVAL
    assert L.topk_attn_k_schedule(100, 4, 1.0, None) == ta.EINVAL
