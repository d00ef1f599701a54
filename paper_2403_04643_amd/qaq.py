"""ctypes binding over libqaq.so: argument marshalling only.

Every step of the method runs inside the library's HIP kernels; PyTorch is used
here for device memory (torch tensors own every buffer, including the cache
arena) and for the stream the kernels are enqueued on.  There is no CPU
fallback: `load()` raises if the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqaq.so")
TILE = 256

OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_HIP, ERR_NEED_ORIGINAL = 0, -1, -2, -3, -4


class Config(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("max_tokens", C.c_int32),
        ("bit_set", C.c_int32 * 5), ("n_bits", C.c_int32),
        ("outlier_frac", C.c_float), ("n_outlier_per_side", C.c_int32),
        ("window", C.c_int32), ("window_store", C.c_int32),
        ("sigma_s_max", C.c_double), ("sigma_x_max", C.c_double),
        ("qnorm2", C.POINTER(C.c_float)),
        ("outlier_thresholds", C.POINTER(C.c_float)),
    ]


class Stats(C.Structure):
    _fields_ = [
        ("tokens", C.c_int64), ("hist_k", C.c_int64 * 5), ("hist_v", C.c_int64 * 5),
        ("code_bytes", C.c_int64), ("layout_code_bytes", C.c_int64), ("meta_bytes", C.c_int64),
        ("fp16_bytes", C.c_int64), ("refused_upgrades", C.c_int64), ("served_upgrades", C.c_int64),
        ("update_handovers", C.c_int64),
    ]


# name -> (restype, argtypes); the names are those declared in include/qaq.h
_vp, _i32, _u8p, _f32p = C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p
SIGNATURES = {
    "qaq_arena_bytes": (C.c_size_t, [C.POINTER(Config)]),
    "qaq_create": (C.c_int, [C.POINTER(Config), _vp, C.c_size_t, C.POINTER(_vp)]),
    "qaq_destroy": (C.c_int, [_vp]),
    "qaq_reset": (C.c_int, [_vp]),
    "qaq_length": (C.c_int, [_vp, C.POINTER(C.c_int32)]),
    "qaq_lengths": (C.c_int, [_vp, C.POINTER(C.c_int32)]),
    "qaq_set_shortfall": (C.c_int, [_vp, C.POINTER(C.c_int32)]),
    "qaq_set_sigmas": (C.c_int, [_vp, C.c_double, C.c_double]),
    "qaq_thresholds": (C.c_int, [_vp, _i32, C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "qaq_quantize_append": (C.c_int, [_vp, _vp, _vp, _i32, _u8p, _u8p, _vp]),
    "qaq_select_bits": (C.c_int, [_vp, _f32p, _u8p, _u8p, _vp]),
    "qaq_requantize": (C.c_int, [_vp, _u8p, _u8p, _vp, _vp, _i32, _vp]),
    "qaq_decode_update": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp, _i32, _u8p, _u8p, _vp]),
    "qaq_prefill_window": (C.c_int, [_vp, _vp, _i32, _vp, _i32, _f32p, _vp]),
    "qaq_quantize_append_selected": (C.c_int, [_vp, _vp, _vp, _i32, _u8p, _u8p, _vp]),
    "qaq_host_alloc": (C.c_int, [C.c_size_t, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]),
    "qaq_host_free": (C.c_int, [_vp]),
    "qaq_profile_begin": (C.c_int, [_vp, _i32]),
    "qaq_profile_read": (C.c_int, [_vp, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_int32)]),
    "qaq_stream_read": (C.c_int, [_vp, C.c_size_t, _vp, _vp]),
    "qaq_stream_copy": (C.c_int, [_vp, _vp, C.c_size_t, _vp]),
    "qaq_decode_attention": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _f32p, _vp]),
    "qaq_decode_attention_static": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _i32, _f32p, _vp]),
    "qaq_static_scratch_limit": (C.c_size_t, []),
    "qaq_dequantize": (C.c_int, [_vp, _i32, _i32, _vp, _vp, _vp]),
    "qaq_export_canonical": (C.c_int, [_vp, _i32, _u8p, _vp, _u8p, _vp, _u8p, _vp]),
    "qaq_stats": (C.c_int, [_vp, C.POINTER(Stats), _vp]),
    "qaq_outliers_per_side": (C.c_int, [C.POINTER(Config)]),
    "qaq_last_error": (C.c_char_p, []),
    "qaq_debug_field": (C.c_int, [_i32] * 10 + [C.POINTER(C.c_uint32), C.POINTER(C.c_int32), C.POINTER(C.c_uint32)]),
    "qaq_debug_tile_capacity": (C.c_uint32, [_i32, _i32]),
}

_lib = None


class QaqError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libqaq error {code}: {msg}")
        self.code = code


def load() -> C.CDLL:
    """Load libqaq.so (built by __graft_entry__.build()).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python __graft_entry__.py`; "
                               "there is no fallback path")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(rc: int) -> None:
    if rc != OK:
        raise QaqError(rc, load().qaq_last_error().decode())


def make_config(batch, n_q_heads, n_kv_heads, head_dim, max_tokens, qnorm2: Sequence[float],
                bit_set=(2, 3, 4, 8), outlier_frac=0.01, n_outlier_per_side=-1, window=5,
                sigma_s_max=1e-3, sigma_x_max=1e-2, window_fp16=False, window_bf16=False,
                outlier_thresholds=None):
    cfg = Config()
    cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.max_tokens = batch, n_q_heads, n_kv_heads, head_dim, max_tokens
    for i, b in enumerate(bit_set):
        cfg.bit_set[i] = int(b)
    cfg.n_bits = len(bit_set)
    cfg.outlier_frac = outlier_frac
    cfg.n_outlier_per_side = n_outlier_per_side
    cfg.window = window
    assert not (window_fp16 and window_bf16)
    cfg.window_store = 1 if window_fp16 else 2 if window_bf16 else 0
    cfg.sigma_s_max, cfg.sigma_x_max = sigma_s_max, sigma_x_max
    arr = (C.c_float * len(qnorm2))(*[float(x) for x in qnorm2])
    cfg.qnorm2 = C.cast(arr, C.POINTER(C.c_float))
    cfg._keepalive = arr
    if outlier_thresholds is not None:     # [2 (K, V)][n_kv_heads][2 (lo, hi)]
        flat = [float(x) for side in outlier_thresholds for pair in side for x in pair]
        assert len(flat) == 4 * n_kv_heads
        arr2 = (C.c_float * len(flat))(*flat)
        cfg.outlier_thresholds = C.cast(arr2, C.POINTER(C.c_float))
        cfg._keepalive2 = arr2
    return cfg


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, HostBuffer):
        return t.dev_ptr
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


class HostBuffer:
    """Page-locked host memory the device can address (qaq_host_alloc): `array` is the CPU's
    view (numpy, the given dtype and shape), `dev_ptr` the address to hand to the library as
    an unquantized copy."""

    def __init__(self, shape, dtype):
        import numpy as np
        self.lib = load()
        nbytes = int(np.prod(shape)) * np.dtype(dtype).itemsize
        h, d = C.c_void_p(), C.c_void_p()
        _check(self.lib.qaq_host_alloc(nbytes, C.byref(h), C.byref(d)))
        self.host_ptr, self.dev_ptr, self.shape = h.value, d.value, tuple(shape)
        self.array = np.frombuffer((C.c_char * nbytes).from_address(h.value), dtype=dtype).reshape(shape)

    def data_ptr(self):
        return self.dev_ptr

    def close(self):
        if getattr(self, "host_ptr", None):
            self.array = None
            self.lib.qaq_host_free(self.host_ptr)
            self.host_ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Cache:
    """A quantized KV cache of one layer.  Methods mirror the C entry points."""

    def __init__(self, cfg: Config, device="cuda:0"):
        import torch
        self.lib = load()
        self.cfg = cfg
        self.device = torch.device(device)
        n = self.lib.qaq_arena_bytes(C.byref(cfg))
        if n == 0:
            raise QaqError(ERR_INVALID_ARG, self.lib.qaq_last_error().decode())
        self.arena = torch.empty(n + 256, dtype=torch.uint8, device=self.device)
        off = (-self.arena.data_ptr()) % 256
        self.arena_bytes = n
        self._base = self.arena.data_ptr() + off
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(self.lib.qaq_create(C.byref(cfg), self._base, n, C.byref(h)))
        self.h = h
        self.n_o = self.lib.qaq_outliers_per_side(C.byref(cfg))

    def close(self):
        if getattr(self, "h", None):
            self.lib.qaq_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- bookkeeping ---------------------------------------------------------------
    def length(self) -> int:
        n = C.c_int32()
        _check(self.lib.qaq_length(self.h, C.byref(n)))
        return n.value

    def lengths(self):
        n = (C.c_int32 * self.cfg.batch)()
        _check(self.lib.qaq_lengths(self.h, n))
        return list(n)

    def set_shortfall(self, shortfall):
        s = (C.c_int32 * self.cfg.batch)(*[int(x) for x in shortfall])
        if len(shortfall) != self.cfg.batch:
            raise ValueError("one shortfall per sequence")
        _check(self.lib.qaq_set_shortfall(self.h, s))

    def reset(self):
        _check(self.lib.qaq_reset(self.h))

    def set_sigmas(self, sigma_s_max: float, sigma_x_max: float):
        _check(self.lib.qaq_set_sigmas(self.h, sigma_s_max, sigma_x_max))

    def thresholds(self, T: int):
        tau = (C.c_float * self.cfg.n_kv_heads)()
        cv = C.c_float()
        _check(self.lib.qaq_thresholds(self.h, T, tau, C.byref(cv)))
        return list(tau), cv.value

    # -- the five calls of the hot path -----------------------------------------------
    def quantize_append(self, k, v, k_bits=None, v_bits=None):
        """k, v: fp16 [B, Hkv, n_new, D]; bits: uint8 [B, Hkv, n_new] or None (= widest)."""
        n_new = k.shape[2]
        _check(self.lib.qaq_quantize_append(self.h, _ptr(k), _ptr(v), n_new, _ptr(k_bits), _ptr(v_bits), _stream()))

    def select_bits(self, scores=None):
        """scores: fp32 [B, Hq, T] or None.  Returns (k_bits, v_bits) uint8 [B, Hkv, T]."""
        import torch
        T = self.length()
        shape = (self.cfg.batch, self.cfg.n_kv_heads, T)
        kb = torch.empty(shape, dtype=torch.uint8, device=self.device)
        vb = torch.empty(shape, dtype=torch.uint8, device=self.device)
        if scores is not None:
            assert tuple(scores.shape) == (self.cfg.batch, self.cfg.n_q_heads, T), "scores must be [B, Hq, T]"
        _check(self.lib.qaq_select_bits(self.h, _ptr(scores), _ptr(kb), _ptr(vb), _stream()))
        return kb, vb

    def select_bits_into(self, scores, kb, vb):
        _check(self.lib.qaq_select_bits(self.h, _ptr(scores), _ptr(kb), _ptr(vb), _stream()))

    def requantize(self, k_bits, v_bits, k_orig=None, v_orig=None):
        """bits: uint8 [B, Hkv, T] or None; originals: fp16 [B, Hkv, >=T, D] or None."""
        src = k_orig if k_orig is not None else v_orig
        n_orig = src.shape[2] if src is not None else 0
        if k_orig is not None and v_orig is not None:
            assert k_orig.shape[2] == v_orig.shape[2]
        _check(self.lib.qaq_requantize(self.h, _ptr(k_bits), _ptr(v_bits), _ptr(k_orig), _ptr(v_orig), n_orig, _stream()))

    def decode_update(self, scores, k_new, v_new, k_orig=None, v_orig=None, want_bits=False):
        """The part of a decode step after the attention, in one call: scores fp32
        [B, Hq, T+1]; k_new, v_new fp16 [B, Hkv, D]; originals fp16 [B, Hkv, >=T+1, D] or
        None.  Returns (k_bits, v_bits) uint8 [B, Hkv, T+1] if want_bits."""
        import torch
        cfg = self.cfg
        src = k_orig if k_orig is not None else v_orig
        n_orig = src.shape[2] if src is not None else 0
        kb = vb = None
        if want_bits:
            T1 = self.length() + 1
            kb = torch.empty((cfg.batch, cfg.n_kv_heads, T1), dtype=torch.uint8, device="cuda")
            vb = torch.empty_like(kb)
        _check(self.lib.qaq_decode_update(self.h, _ptr(scores), _ptr(k_new), _ptr(v_new), _ptr(k_orig), _ptr(v_orig),
                                          n_orig, _ptr(kb), _ptr(vb), _stream()))
        return kb, vb

    def prefill_window(self, q_last, k, scores_out=None):
        """Prompt encoding: q_last fp16 [B, Hq, n, D] (queries of the last n prompt positions),
        k fp16 [B, Hkv, T, D].  The last n causal score rows become the window.
        Returns them: fp32 [n, B, Hq, T] (entries of a row past its length are 0)."""
        import torch
        cfg = self.cfg
        n, T = q_last.shape[2], k.shape[2]
        if scores_out is None:
            scores_out = torch.empty((n, cfg.batch, cfg.n_q_heads, T), dtype=torch.float32, device=self.device)
        _check(self.lib.qaq_prefill_window(self.h, _ptr(q_last), n, _ptr(k), T, _ptr(scores_out), _stream()))
        return scores_out

    def quantize_append_selected(self, k, v, want_bits=False):
        """k, v: fp16 [B, Hkv, n_new, D], appended at the widths the rules give from the window
        as it stands.  Returns (k_bits, v_bits) uint8 [B, Hkv, n_new] if want_bits."""
        import torch
        cfg = self.cfg
        n_new = k.shape[2]
        kb = vb = None
        if want_bits:
            kb = torch.empty((cfg.batch, cfg.n_kv_heads, n_new), dtype=torch.uint8, device=self.device)
            vb = torch.empty_like(kb)
        _check(self.lib.qaq_quantize_append_selected(self.h, _ptr(k), _ptr(v), n_new, _ptr(kb), _ptr(vb), _stream()))
        return kb, vb

    def profile_begin(self, max_calls: int):
        _check(self.lib.qaq_profile_begin(self.h, max_calls))
        self._prof_cap = max_calls

    def profile_read(self):
        """Returns (ms of the per-tile kernel, ms of the merge kernel), one list entry per
        profiled call."""
        n = C.c_int32()
        a = (C.c_float * max(self._prof_cap, 1))()
        b = (C.c_float * max(self._prof_cap, 1))()
        _check(self.lib.qaq_profile_read(self.h, a, b, C.byref(n)))
        return list(a[: n.value]), list(b[: n.value])

    def decode_attention_static(self, q, k_new, v_new, out, scores_out=None):
        """qaq_decode_attention_static: every buffer is the caller's, nothing is allocated."""
        import torch
        _check(self.lib.qaq_decode_attention_static(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                    1 if out.dtype == torch.float32 else 0, _ptr(scores_out), _stream()))

    def decode_attention(self, q, k_new=None, v_new=None, out=None, scores_out=None, want_scores=False, out_fp32=True):
        """q: fp16 [B, Hq, D]; k_new, v_new: fp16 [B, Hkv, D] or None.
        Returns (X [B, Hq, D], scores [B, Hq, T(+1)] or None)."""
        import torch
        cfg = self.cfg
        if out is None:
            out = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim),
                              dtype=torch.float32 if out_fp32 else torch.float16, device=self.device)
        if scores_out is None and want_scores:
            scores_out = torch.empty((cfg.batch, cfg.n_q_heads, self.length() + (k_new is not None)),
                                     dtype=torch.float32, device=self.device)
        _check(self.lib.qaq_decode_attention(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                             1 if out.dtype == torch.float32 else 0, _ptr(scores_out), _stream()))
        return out, scores_out

    def dequantize(self, t0=0, t1=None, want_k=True, want_v=True):
        import torch
        cfg = self.cfg
        t1 = self.length() if t1 is None else t1
        shape = (cfg.batch, cfg.n_kv_heads, t1 - t0, cfg.head_dim)
        k = torch.empty(shape, dtype=torch.float16, device=self.device) if want_k else None
        v = torch.empty(shape, dtype=torch.float16, device=self.device) if want_v else None
        _check(self.lib.qaq_dequantize(self.h, t0, t1, _ptr(k), _ptr(v), _stream()))
        return k, v

    # -- observability ---------------------------------------------------------------
    def export_canonical(self, side: int):
        """Returns dict(bits, minmax, oidx, oval, codes) of device tensors, by position."""
        import torch
        cfg = self.cfg
        T = self.length()
        B, H, D, k = cfg.batch, cfg.n_kv_heads, cfg.head_dim, 2 * self.n_o
        dev = self.device
        out = dict(
            bits=torch.empty((B, H, T), dtype=torch.uint8, device=dev),
            minmax=torch.empty((B, H, T, 2), dtype=torch.float16, device=dev),
            oidx=torch.empty((B, H, T, max(k, 1)), dtype=torch.uint8, device=dev),
            oval=torch.empty((B, H, T, max(k, 1)), dtype=torch.float16, device=dev),
            codes=torch.empty((B, H, T, D), dtype=torch.uint8, device=dev),
        )
        _check(self.lib.qaq_export_canonical(self.h, side, _ptr(out["bits"]), _ptr(out["minmax"]),
                                             _ptr(out["oidx"]) if k else None, _ptr(out["oval"]) if k else None,
                                             _ptr(out["codes"]), _stream()))
        if k == 0:
            out["oidx"] = out["oidx"][..., :0]
            out["oval"] = out["oval"][..., :0]
        return out

    def stats(self) -> Stats:
        st = Stats()
        _check(self.lib.qaq_stats(self.h, C.byref(st), _stream()))
        return st


def debug_field(side, D, counts, bf, idx, d):
    """Host-only layout query: (byte offset of the 32-bit word, bit shift, end of regions)."""
    lib = load()
    off, sh, end = C.c_uint32(), C.c_int32(), C.c_uint32()
    n3, n2, n4, n8, n1 = counts
    _check(lib.qaq_debug_field(side, D, n3, n2, n4, n8, n1, bf, idx, d, C.byref(off), C.byref(sh), C.byref(end)))
    return off.value, sh.value, end.value
