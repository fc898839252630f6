"""ctypes binding of libtopk_attn.so: argument marshalling only.

Function names follow include/topk_attn.h one to one.  PyTorch supplies device
memory (tensors whose data_ptr() is handed over) and the HIP stream; all
computation happens in the library's kernels.  There is no fallback: if the
shared library is missing, importing any entry point raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtopk_attn.so")

OK, EINVAL, ECAPACITY, EUNSUPPORTED, EDEVICE, ENOMEM, ESCRATCH = range(7)
F32, F16, BF16 = 0, 1, 2
PATH_AUTO, PATH_FULL, PATH_FILTER, PATH_INDEX, PATH_PAGES = 0, 1, 2, 3, 4
INDEX_NONE, INDEX_INT8, INDEX_PAGES = 0, 1, 2

EXPORTS = [
    "topk_attn_kv_bytes", "topk_attn_workspace_bytes", "topk_attn_create", "topk_attn_append_kv", "topk_attn_append_step",
    "topk_attn_decode", "topk_attn_decode_static", "topk_attn_decode_window", "topk_attn_decode_multi", "topk_attn_decode_layers", "topk_attn_k_schedule", "topk_attn_scores", "topk_attn_length", "topk_attn_reset", "topk_attn_set_path",
    "topk_attn_last_fallbacks", "topk_attn_set_page_bound_scale", "topk_attn_last_pages_read", "topk_attn_last_selection_records", "topk_attn_debug_read_workspace", "topk_attn_debug_read_workspace_dims", "topk_attn_debug_force_redo", "topk_attn_set_scan_timing", "topk_attn_scan_time", "topk_attn_read_probe", "topk_attn_build_id", "topk_attn_strerror", "topk_attn_destroy",
]


class Config(ctypes.Structure):
    """Mirror of topk_attn_config."""
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("n_layers", ctypes.c_int32),
        ("n_seqs", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("max_tokens", ctypes.c_int64),
        ("max_k", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("device", ctypes.c_int32),
        ("max_window", ctypes.c_int32),
        ("max_queries", ctypes.c_int32),
        ("index_kind", ctypes.c_int32),
        ("kv_storage", ctypes.c_void_p),
        ("kv_bytes", ctypes.c_size_t),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_06766_amd.build` "
                "(hipcc, gfx950); there is no fallback path")
        # PyTorch ships the HIP runtime that owns the tensors handed to the library; load it
        # first so that the library binds to that same runtime instead of a second copy.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        cfgp = ctypes.POINTER(Config)
        L.topk_attn_kv_bytes.argtypes = [cfgp]
        L.topk_attn_kv_bytes.restype = sz
        L.topk_attn_workspace_bytes.argtypes = [cfgp]
        L.topk_attn_workspace_bytes.restype = sz
        L.topk_attn_create.argtypes = [cfgp, ctypes.POINTER(vp)]
        L.topk_attn_create.restype = i32
        L.topk_attn_append_kv.argtypes = [vp, i32, i32, vp, vp, i64, i64, i64, vp]
        L.topk_attn_append_kv.restype = i32
        L.topk_attn_append_step.argtypes = [vp, i32, vp, vp, i64, vp]
        L.topk_attn_append_step.restype = i32
        L.topk_attn_decode.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp]
        L.topk_attn_decode.restype = i32
        L.topk_attn_decode_static.argtypes = [vp, i32, vp, i32, vp, vp, vp, vp, vp]
        L.topk_attn_decode_static.restype = i32
        L.topk_attn_decode_window.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp, vp, vp]
        L.topk_attn_decode_window.restype = i32
        L.topk_attn_decode_multi.argtypes = [vp, i32, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.topk_attn_decode_multi.restype = i32
        L.topk_attn_decode_layers.argtypes = [vp, i32, i32, vp, ctypes.POINTER(ctypes.c_int32), i32, vp, vp, vp, vp, vp]
        L.topk_attn_decode_layers.restype = i32
        L.topk_attn_k_schedule.argtypes = [i64, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_int32)]
        L.topk_attn_k_schedule.restype = i32
        L.topk_attn_scores.argtypes = [vp, i32, vp, vp, vp]
        L.topk_attn_scores.restype = i32
        L.topk_attn_length.argtypes = [vp, i32, i32]
        L.topk_attn_length.restype = i64
        L.topk_attn_reset.argtypes = [vp, i32, i32, vp]
        L.topk_attn_reset.restype = i32
        L.topk_attn_set_path.argtypes = [vp, i32]
        L.topk_attn_set_path.restype = i32
        L.topk_attn_last_fallbacks.argtypes = [vp, ctypes.POINTER(i32)]
        L.topk_attn_last_fallbacks.restype = i32
        L.topk_attn_set_page_bound_scale.argtypes = [vp, ctypes.c_float]
        L.topk_attn_set_page_bound_scale.restype = i32
        L.topk_attn_last_pages_read.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.topk_attn_last_pages_read.restype = i32
        L.topk_attn_last_selection_records.argtypes = [vp, ctypes.POINTER(ctypes.c_uint32)]
        L.topk_attn_last_selection_records.restype = i32
        L.topk_attn_debug_read_workspace.argtypes = [vp, ctypes.c_char_p, vp, ctypes.c_size_t]
        L.topk_attn_debug_read_workspace.restype = i32
        L.topk_attn_debug_read_workspace_dims.argtypes = [vp, ctypes.POINTER(i32)]
        L.topk_attn_debug_read_workspace_dims.restype = i32
        L.topk_attn_debug_force_redo.argtypes = [vp, i32]
        L.topk_attn_debug_force_redo.restype = i32
        L.topk_attn_set_scan_timing.argtypes = [vp, i32]
        L.topk_attn_set_scan_timing.restype = i32
        L.topk_attn_scan_time.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        L.topk_attn_scan_time.restype = i32
        L.topk_attn_read_probe.argtypes = [vp, sz, vp, vp]
        L.topk_attn_read_probe.restype = i32
        L.topk_attn_build_id.argtypes = []
        L.topk_attn_build_id.restype = ctypes.c_char_p
        L.topk_attn_strerror.argtypes = [i32]
        L.topk_attn_strerror.restype = ctypes.c_char_p
        L.topk_attn_destroy.argtypes = [vp]
        L.topk_attn_destroy.restype = i32
        _lib = L
    return _lib


class TopkAttnError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {topk_attn_strerror(code)} (code {code})")


def _check(code: int, where: str) -> None:
    if code != OK:
        raise TopkAttnError(code, where)


def make_config(n_layers, n_seqs, n_q_heads, n_kv_heads, head_dim, max_tokens, max_k, dtype, device=0,
                kv_storage=0, kv_bytes=0, workspace=0, workspace_bytes=0, max_window=0, max_queries=0,
                index_kind=0) -> Config:
    return Config(ctypes.sizeof(Config), n_layers, n_seqs, n_q_heads, n_kv_heads, head_dim, max_tokens,
                  max_k, dtype, device, max_window, max_queries, index_kind, kv_storage, kv_bytes, workspace,
                  workspace_bytes)


def topk_attn_strerror(code: int) -> str:
    return lib().topk_attn_strerror(code).decode()


def topk_attn_build_id() -> str:
    return lib().topk_attn_build_id().decode()


def topk_attn_kv_bytes(cfg: Config) -> int:
    return int(lib().topk_attn_kv_bytes(ctypes.byref(cfg)))


def topk_attn_workspace_bytes(cfg: Config) -> int:
    return int(lib().topk_attn_workspace_bytes(ctypes.byref(cfg)))


def topk_attn_create(cfg: Config) -> int:
    """Returns the opaque handle (an integer address); raises TopkAttnError."""
    h = ctypes.c_void_p()
    _check(lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)), "topk_attn_create")
    return h.value


def topk_attn_destroy(h: int) -> None:
    _check(lib().topk_attn_destroy(h), "topk_attn_destroy")


def topk_attn_append_kv(h, layer, seq, k_new_ptr, v_new_ptr, n_new, token_stride, head_stride, stream=0):
    _check(lib().topk_attn_append_kv(h, layer, seq, k_new_ptr, v_new_ptr, n_new, token_stride, head_stride,
                                     stream), "topk_attn_append_kv")


def topk_attn_append_step(h, layer, k_new_ptr, v_new_ptr, n_new, stream=0):
    _check(lib().topk_attn_append_step(h, layer, k_new_ptr, v_new_ptr, n_new, stream), "topk_attn_append_step")


def topk_attn_decode(h, layer, q_ptr, k, out_ptr, idx_ptr=0, vals_ptr=0, lse_ptr=0, stream=0):
    _check(lib().topk_attn_decode(h, layer, q_ptr, k, out_ptr, idx_ptr or None, vals_ptr or None,
                                  lse_ptr or None, stream), "topk_attn_decode")


def topk_attn_decode_static(h, layer, q_ptr, k, out_ptr, idx_ptr=0, vals_ptr=0, lse_ptr=0, stream=0):
    _check(lib().topk_attn_decode_static(h, layer, q_ptr, k, out_ptr, idx_ptr or None, vals_ptr or None,
                                         lse_ptr or None, stream), "topk_attn_decode_static")


def topk_attn_decode_window(h, layer, q_ptr, k, window, out_ptr, idx_ptr=0, vals_ptr=0, lse_ptr=0, stream=0):
    _check(lib().topk_attn_decode_window(h, layer, q_ptr, k, window, out_ptr, idx_ptr or None, vals_ptr or None,
                                         lse_ptr or None, stream), "topk_attn_decode_window")


def topk_attn_decode_multi(h, layer, q_ptr, n_queries, causal, k, window, out_ptr, idx_ptr=0, vals_ptr=0, lse_ptr=0,
                           stream=0):
    _check(lib().topk_attn_decode_multi(h, layer, q_ptr, n_queries, 1 if causal else 0, k, window, out_ptr,
                                        idx_ptr or None, vals_ptr or None, lse_ptr or None, stream),
           "topk_attn_decode_multi")


def topk_attn_decode_layers(h, layer0, ks, q_ptr, window, out_ptr, idx_ptr=0, vals_ptr=0, lse_ptr=0, stream=0):
    """ks: per-layer k (sequence of ints) for layers layer0 .. layer0 + len(ks) - 1."""
    arr = (ctypes.c_int32 * max(1, len(ks)))(*ks)
    _check(lib().topk_attn_decode_layers(h, layer0, len(ks), q_ptr, arr, window, out_ptr, idx_ptr or None,
                                         vals_ptr or None, lse_ptr or None, stream), "topk_attn_decode_layers")


def topk_attn_k_schedule(total_k: int, n_layers: int, last_over_first: float = 1.0):
    """Per-layer k with a fixed total budget (host only); returns a list of n_layers ints."""
    buf = (ctypes.c_int32 * max(1, n_layers))()
    _check(lib().topk_attn_k_schedule(total_k, n_layers, last_over_first, buf), "topk_attn_k_schedule")
    return list(buf)[:n_layers]


def topk_attn_scores(h, layer, q_ptr, scores_ptr, stream=0):
    _check(lib().topk_attn_scores(h, layer, q_ptr, scores_ptr, stream), "topk_attn_scores")


def topk_attn_length(h, layer, seq) -> int:
    return int(lib().topk_attn_length(h, layer, seq))


def topk_attn_reset(h, layer, seq, stream=0):
    _check(lib().topk_attn_reset(h, layer, seq, stream), "topk_attn_reset")


def topk_attn_set_path(h, path):
    _check(lib().topk_attn_set_path(h, path), "topk_attn_set_path")


def topk_attn_last_fallbacks(h) -> int:
    n = ctypes.c_int(0)
    _check(lib().topk_attn_last_fallbacks(h, ctypes.byref(n)), "topk_attn_last_fallbacks")
    return n.value


def topk_attn_set_page_bound_scale(h, beta: float):
    _check(lib().topk_attn_set_page_bound_scale(h, beta), "topk_attn_set_page_bound_scale")


def topk_attn_last_pages_read(h):
    """(pages read by the last decode's key scan, pages cached); sync the stream first."""
    a, b = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().topk_attn_last_pages_read(h, ctypes.byref(a), ctypes.byref(b)), "topk_attn_last_pages_read")
    return a.value, b.value


def topk_attn_last_selection_records(h, n_heads_total: int):
    """[n_heads_total][4] (state, certain, to pick, in the boundary bin) of the last decode; sync the stream first."""
    buf = (ctypes.c_uint32 * (4 * n_heads_total))()
    _check(lib().topk_attn_last_selection_records(h, buf), "topk_attn_last_selection_records")
    return [tuple(buf[4 * i:4 * i + 4]) for i in range(n_heads_total)]


def topk_attn_debug_read_workspace(h, name: str, dtype, count: int):
    """The first `count` elements (numpy `dtype`) of a named per-call array of the workspace; sync the stream first."""
    import numpy as np
    a = np.empty(count, dtype=dtype)
    _check(lib().topk_attn_debug_read_workspace(h, name.encode(), a.ctypes.data, a.nbytes), "topk_attn_debug_read_workspace")
    return a


def topk_attn_debug_read_workspace_dims(h):
    """(cand_cap, bnd_cap, hist_cap, most segments, segments and entries per segment of the last filtered decode)."""
    d = (ctypes.c_int32 * 6)()
    _check(lib().topk_attn_debug_read_workspace_dims(h, d), "topk_attn_debug_read_workspace_dims")
    return tuple(d)


def topk_attn_debug_force_redo(h, enable: bool):
    _check(lib().topk_attn_debug_force_redo(h, 1 if enable else 0), "topk_attn_debug_force_redo")


def topk_attn_set_scan_timing(h, enable: bool):
    _check(lib().topk_attn_set_scan_timing(h, 1 if enable else 0), "topk_attn_set_scan_timing")


def topk_attn_scan_time(h):
    """(total_ms, n_calls) of the key-scan kernel since the last read; sync the stream first."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int(0)
    _check(lib().topk_attn_scan_time(h, ctypes.byref(ms), ctypes.byref(n)), "topk_attn_scan_time")
    return ms.value, n.value


def topk_attn_read_probe(src_ptr, nbytes, sink_ptr, stream=0):
    _check(lib().topk_attn_read_probe(src_ptr, nbytes, sink_ptr, stream), "topk_attn_read_probe")


# --------------------------------------------------------------------------
# Convenience owner of the torch allocations a handle borrows (marshalling only).
# --------------------------------------------------------------------------
class TopkAttnCache:
    """Allocates kv_storage/workspace as torch tensors and wraps the handle."""

    def __init__(self, n_layers, n_seqs, n_q_heads, n_kv_heads, head_dim, max_tokens, max_k, dtype, device=0,
                 max_window=0, max_queries=0, index_kind=0):
        import torch
        self.torch = torch
        self.shape = (n_layers, n_seqs, n_q_heads, n_kv_heads, head_dim, max_tokens, max_k, dtype)
        self.dtype = dtype
        self.device = torch.device("cuda", device)
        cfg = make_config(n_layers, n_seqs, n_q_heads, n_kv_heads, head_dim, max_tokens, max_k, dtype, device,
                          max_window=max_window, max_queries=max_queries, index_kind=index_kind)
        kvb, wsb = topk_attn_kv_bytes(cfg), topk_attn_workspace_bytes(cfg)
        if kvb == 0 or wsb == 0:
            h = ctypes.c_void_p()
            _check(lib().topk_attn_create(ctypes.byref(cfg), ctypes.byref(h)), "topk_attn_create")
        self.kv = torch.empty(kvb, dtype=torch.uint8, device=self.device)
        self.ws = torch.empty(wsb, dtype=torch.uint8, device=self.device)
        cfg.kv_storage, cfg.kv_bytes = self.kv.data_ptr(), kvb
        cfg.workspace, cfg.workspace_bytes = self.ws.data_ptr(), wsb
        torch.cuda.synchronize(self.device)
        self.h = topk_attn_create(cfg)
        self.cfg = cfg

    def torch_dtype(self):
        t = self.torch
        return {F32: t.float32, F16: t.float16, BF16: t.bfloat16}[self.dtype]

    def _stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def append(self, layer, seq, k_new, v_new, head_major=False):
        """k_new/v_new: [n, Hkv, d] (token-major) or [Hkv, n, d] (head_major) device tensors."""
        assert k_new.is_cuda and v_new.is_cuda and k_new.dtype == self.torch_dtype()
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
        d = k_new.shape[-1]
        if head_major:
            n = k_new.shape[1]
            ts, hs = d, n * d
        else:
            n = k_new.shape[0]
            ts, hs = k_new.shape[1] * d, d
        topk_attn_append_kv(self.h, layer, seq, k_new.data_ptr(), v_new.data_ptr(), n, ts, hs, self._stream())

    def append_step(self, layer, k_new, v_new):
        """k_new/v_new: [B, n, Hkv, d] device tensors: n tokens for every sequence of the layer."""
        assert k_new.is_cuda and v_new.is_cuda and k_new.dtype == self.torch_dtype()
        assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.shape == v_new.shape
        topk_attn_append_step(self.h, layer, k_new.data_ptr(), v_new.data_ptr(), k_new.shape[1], self._stream())

    def decode(self, layer, q, k, want_idx=True, want_vals=True, want_lse=True, window=0):
        """q [B, Hq, d] device tensor -> (out, idx, vals, lse) device tensors (None if not wanted)."""
        t = self.torch
        B, Hq, d = q.shape
        assert q.is_cuda and q.is_contiguous() and q.dtype == self.torch_dtype()
        out = t.empty((B, Hq, d), dtype=t.float32, device=self.device)
        idx = t.empty((B, Hq, k), dtype=t.int32, device=self.device) if want_idx else None
        vals = t.empty((B, Hq, k), dtype=t.float32, device=self.device) if want_vals else None
        lse = t.empty((B, Hq), dtype=t.float32, device=self.device) if want_lse else None
        args = (out.data_ptr(), idx.data_ptr() if want_idx else 0, vals.data_ptr() if want_vals else 0,
                lse.data_ptr() if want_lse else 0, self._stream())
        if window:
            topk_attn_decode_window(self.h, layer, q.data_ptr(), k, window, *args)
        else:
            topk_attn_decode(self.h, layer, q.data_ptr(), k, *args)
        return out, idx, vals, lse

    def decode_multi(self, layer, q, k, causal=True, window=0, want_idx=True, want_vals=True, want_lse=True):
        """q [B, M, Hq, d] device tensor -> (out [B, M, Hq, d], idx, vals [B, M, Hq, k], lse [B, M, Hq])."""
        t = self.torch
        B, M, Hq, d = q.shape
        assert q.is_cuda and q.is_contiguous() and q.dtype == self.torch_dtype()
        out = t.empty((B, M, Hq, d), dtype=t.float32, device=self.device)
        idx = t.empty((B, M, Hq, k), dtype=t.int32, device=self.device) if want_idx else None
        vals = t.empty((B, M, Hq, k), dtype=t.float32, device=self.device) if want_vals else None
        lse = t.empty((B, M, Hq), dtype=t.float32, device=self.device) if want_lse else None
        topk_attn_decode_multi(self.h, layer, q.data_ptr(), M, causal, k, window, out.data_ptr(),
                               idx.data_ptr() if want_idx else 0, vals.data_ptr() if want_vals else 0,
                               lse.data_ptr() if want_lse else 0, self._stream())
        return out, idx, vals, lse

    def scores(self, layer, q):
        t = self.torch
        B, Hq, _ = q.shape
        s = t.zeros((B, Hq, self.shape[5]), dtype=t.float32, device=self.device)
        topk_attn_scores(self.h, layer, q.data_ptr(), s.data_ptr(), self._stream())
        return s

    def length(self, layer, seq) -> int:
        return topk_attn_length(self.h, layer, seq)

    def reset(self, layer, seq):
        topk_attn_reset(self.h, layer, seq, self._stream())

    def set_path(self, path):
        topk_attn_set_path(self.h, path)

    def last_fallbacks(self) -> int:
        self.torch.cuda.synchronize(self.device)
        return topk_attn_last_fallbacks(self.h)

    def close(self):
        if self.h:
            self.torch.cuda.synchronize(self.device)
            topk_attn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
