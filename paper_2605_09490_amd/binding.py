"""Thin ctypes binding of libtkv.so: same names as the C ABI (include/tkv.h), argument marshalling only.

PyTorch provides device memory, pinned host memory and streams; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtkv.so")

TKV_OK, TKV_EINVAL, TKV_ENOMEM, TKV_ECAPACITY, TKV_ESTATE, TKV_EDEVICE = 0, -1, -2, -3, -4, -5
TKV_F32, TKV_BF16, TKV_F16 = 0, 1, 2
TKV_T2_INT8_ROW, TKV_T2_INT4_G32 = 0, 1
TKV_PREFETCH_WAIT, TKV_PREFETCH_LAZY, TKV_PREFETCH_STREAM = 0, 1, 2
TKV_SCORE_ATTENTION, TKV_SCORE_VATP, TKV_SCORE_REDUNDANCY, TKV_SCORE_COMBINED = 0, 1, 2, 3
TKV_COUNT_TOTAL, TKV_COUNT_ALG1 = 0, 1
STATUS_NAMES = {0: "TKV_OK", -1: "TKV_EINVAL", -2: "TKV_ENOMEM", -3: "TKV_ECAPACITY", -4: "TKV_ESTATE", -5: "TKV_EDEVICE"}

ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class tkv_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("max_tokens", C.c_int32), ("kv_dtype", C.c_int32), ("out_dtype", C.c_int32),
        ("t2_format", C.c_int32),
        ("n_prompt", C.c_int32), ("k_sink", C.c_int32), ("k_window", C.c_int32),
        ("score_scale", C.c_float), ("softmax_scale", C.c_float),
        ("t0_rows", C.c_int32), ("staging_rows", C.c_int32), ("t2_rows", C.c_int32),
        ("host_rows", C.c_int64), ("bounce_bytes", C.c_int64),
        ("prefetch_mode", C.c_int32), ("profile", C.c_int32), ("scorer", C.c_int32), ("device", C.c_int32),
        ("redundancy_weight", C.c_float),
        ("dev_alloc", ALLOC_FN), ("dev_free", FREE_FN), ("pin_alloc", ALLOC_FN), ("pin_free", FREE_FN),
        ("alloc_ctx", C.c_void_p),
    ]


class tkv_policy(C.Structure):
    _fields_ = [("f_t0_ppm", C.c_uint32), ("f_t1_ppm", C.c_uint32), ("f_t2_ppm", C.c_uint32), ("f_t3_ppm", C.c_uint32),
                ("count_rule", C.c_uint32)]


class tkv_stats(C.Structure):
    _fields_ = [
        ("tier_count", C.c_int64 * 4), ("h2d_bytes", C.c_int64), ("d2h_bytes", C.c_int64),
        ("h2d_copies", C.c_int64), ("d2h_copies", C.c_int64), ("h2d_ms", C.c_double), ("d2h_ms", C.c_double),
        ("attn_kernel_ms", C.c_double), ("attn_kernel_launches", C.c_int64),
        ("classify_ms", C.c_double), ("migrate_ms", C.c_double),
        ("attend_waits", C.c_int64), ("lazy_old_reads", C.c_int64), ("n_classify", C.c_int64), ("n_migrate", C.c_int64),
        ("n_rehome", C.c_int64), ("host_rows_used", C.c_int64), ("n_repack", C.c_int64), ("device_bytes", C.c_int64), ("pinned_bytes", C.c_int64),
        ("attn_finish_ms", C.c_double), ("attn_call_ms", C.c_double), ("step_ms", C.c_double), ("steps_timed", C.c_int64),
    ]


# every symbol include/tkv.h declares: name -> (restype, argtypes)
_VP, _I32 = C.c_void_p, C.c_int32
SYMBOLS = {
    "tkv_create": (C.c_int, [C.POINTER(tkv_config), C.POINTER(_VP)]),
    "tkv_destroy": (None, [_VP]),
    "tkv_append": (C.c_int, [_VP, _I32, _VP, _VP, _I32, _VP]),
    "tkv_attend_and_score": (C.c_int, [_VP, _I32, _VP, _VP, _VP]),
    "tkv_attend_and_score_noalloc": (C.c_int, [_VP, _I32, _VP, _VP, _VP]),
    "tkv_attend_and_score_chunk": (C.c_int, [_VP, _I32, _VP, _VP, _I32, _VP]),
    "tkv_decode_step": (C.c_int, [_VP, _VP, _VP, _VP, _VP, _VP]),
    "tkv_set_profile": (C.c_int, [_VP, _I32]),
    "tkv_classify": (C.c_int, [_VP, C.POINTER(tkv_policy), _VP]),
    "tkv_migrate": (C.c_int, [_VP, _VP]),
    "tkv_get_scores": (C.c_int, [_VP, _VP]),
    "tkv_set_scores": (C.c_int, [_VP, _VP]),
    "tkv_get_tiers": (C.c_int, [_VP, _VP]),
    "tkv_get_pending_tiers": (C.c_int, [_VP, _VP]),
    "tkv_set_tiers": (C.c_int, [_VP, _VP]),
    "tkv_get_index_list": (C.c_int, [_VP, _I32, _I32, _VP, C.POINTER(_I32)]),
    "tkv_get_t2_row": (C.c_int, [_VP, _I32, _I32, _I32, _I32, _I32, _VP, _VP]),
    "tkv_get_row": (C.c_int, [_VP, _I32, _I32, _I32, _I32, _I32, _VP]),
    "tkv_wait_prefetch": (C.c_int, [_VP]),
    "tkv_get_stats": (C.c_int, [_VP, C.POINTER(tkv_stats)]),
    "tkv_probe_hbm_read": (C.c_int, [_VP, C.c_size_t, _I32, _VP, C.POINTER(C.c_float)]),
    "tkv_layer_length": (_I32, [_VP, _I32]),
    "tkv_last_error": (C.c_char_p, [_VP]),
    "tkv_tier_counts": (C.c_int, [C.POINTER(tkv_policy), C.c_int64, C.c_int64, C.POINTER(C.c_int64)]),
}

_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree libtkv.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2605_09490_amd.build)")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


class TkvError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


def tier_counts(policy_ppm, m, n_already_evicted=0, count_rule=0):
    lib = load_library()
    pol = tkv_policy(*[int(x) for x in policy_ppm], int(count_rule))
    out = (C.c_int64 * 4)()
    st = lib.tkv_tier_counts(C.byref(pol), int(m), int(n_already_evicted), out)
    if st != TKV_OK:
        raise TkvError(st, "tkv_tier_counts")
    return tuple(int(x) for x in out)


def probe_hbm_read(buf, iters=8, stream=None):
    """GB/s a read-only streaming kernel reaches over the CUDA tensor `buf` (average of `iters` passes)."""
    lib = load_library()
    nbytes = buf.numel() * buf.element_size()
    ms = C.c_float(0.0)
    st = lib.tkv_probe_hbm_read(C.c_void_p(buf.data_ptr()), nbytes, int(iters),
                                C.c_void_p((stream or torch.cuda.current_stream()).cuda_stream), C.byref(ms))
    if st != TKV_OK:
        raise TkvError(st, "tkv_probe_hbm_read")
    return nbytes / (ms.value * 1e-3) / 1e9


class TieredKV:
    """Handle on one tkv_cache.  Methods mirror the C entry points; tensors are torch CUDA tensors."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, head_dim, max_tokens, kv_dtype="bf16",
                 t2_format="int8_row", out_dtype="f32", n_prompt=0, k_sink=4, k_window=128, score_scale=0.0, softmax_scale=0.0,
                 t0_rows=0, staging_rows=0, t2_rows=0, host_rows=0, bounce_bytes=0, prefetch_mode="wait",
                 profile=False, device=0, use_torch_allocator=True, scorer="attention", redundancy_weight=0.0):
        self.lib = load_library()
        self.device = torch.device("cuda", device)
        self.shape = (n_layers, batch, n_q_heads, n_kv_heads, head_dim)
        self.max_tokens = max_tokens
        self.kv_dtype = kv_dtype
        self.t2_format = t2_format
        torch_types = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
        codes = {"f32": TKV_F32, "bf16": TKV_BF16, "f16": TKV_F16}
        self.torch_dtype = torch_types[kv_dtype]
        self.out_torch_dtype = torch_types[out_dtype]
        self._held = {}
        cfg = tkv_config()
        cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim = n_layers, batch, n_q_heads, n_kv_heads, head_dim
        cfg.max_tokens = max_tokens
        cfg.kv_dtype = codes[kv_dtype]
        cfg.out_dtype = codes[out_dtype]
        cfg.t2_format = TKV_T2_INT8_ROW if t2_format == "int8_row" else TKV_T2_INT4_G32
        cfg.n_prompt, cfg.k_sink, cfg.k_window = n_prompt, k_sink, k_window
        cfg.score_scale, cfg.softmax_scale = float(score_scale or 0.0), float(softmax_scale or 0.0)
        cfg.t0_rows, cfg.staging_rows, cfg.t2_rows = t0_rows, staging_rows, t2_rows
        cfg.host_rows, cfg.bounce_bytes = host_rows, bounce_bytes
        cfg.prefetch_mode = {"wait": TKV_PREFETCH_WAIT, "lazy": TKV_PREFETCH_LAZY, "stream": TKV_PREFETCH_STREAM}[prefetch_mode]
        cfg.profile = 1 if profile else 0
        cfg.scorer = {"attention": TKV_SCORE_ATTENTION, "vatp": TKV_SCORE_VATP, "redundancy": TKV_SCORE_REDUNDANCY,
                      "combined": TKV_SCORE_COMBINED}[scorer]
        cfg.redundancy_weight = float(redundancy_weight)
        cfg.device = device
        if use_torch_allocator:
            # PyTorch supplies device and pinned memory; the library only sees raw pointers
            self._alloc_error = ""

            def _dev_alloc(nbytes, _ctx):
                try:
                    t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
                except RuntimeError as e:
                    self._alloc_error = f"device allocation of {int(nbytes)} bytes failed: {str(e)[:200]}"
                    return None
                self._held[t.data_ptr()] = t
                return t.data_ptr()

            def _pin_alloc(nbytes, _ctx):
                try:
                    t = torch.empty(int(nbytes), dtype=torch.uint8, pin_memory=True)
                except RuntimeError as e:
                    self._alloc_error = f"pinned allocation of {int(nbytes)} bytes failed: {str(e)[:200]}"
                    return None
                self._held[t.data_ptr()] = t
                return t.data_ptr()

            def _free(ptr, _ctx):
                self._held.pop(ptr, None)

            self._cbs = (ALLOC_FN(_dev_alloc), FREE_FN(_free), ALLOC_FN(_pin_alloc), FREE_FN(_free))
            cfg.dev_alloc, cfg.dev_free, cfg.pin_alloc, cfg.pin_free = self._cbs
        self._cfg = cfg
        h = C.c_void_p()
        st = self.lib.tkv_create(C.byref(cfg), C.byref(h))
        if st != TKV_OK:
            why = getattr(self, "_alloc_error", "")
            raise TkvError(st, self.lib.tkv_last_error(None).decode() + (f" ({why})" if why else ""))
        self._h = h

    # -- helpers ---------------------------------------------------------------------------------
    def _check(self, st):
        if st != TKV_OK:
            raise TkvError(st, self.lib.tkv_last_error(self._h).decode())

    @staticmethod
    def _stream(stream):
        if stream is None:
            stream = torch.cuda.current_stream()
        return C.c_void_p(stream.cuda_stream)

    def _dev_tensor(self, t, shape, dtype=None):
        assert t.is_cuda and t.dtype == (dtype or self.torch_dtype) and t.is_contiguous() and tuple(t.shape) == tuple(shape), \
            (t.device, t.dtype, t.shape, shape)
        return C.c_void_p(t.data_ptr())

    def close(self):
        if getattr(self, "_h", None):
            self.lib.tkv_destroy(self._h)
            self._h = None
            self._held.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the hot path ------------------------------------------------------------------------------
    def append(self, layer, k, v, stream=None):
        L, B, Hq, Hkv, D = self.shape
        n_new = k.shape[1]
        self._check(self.lib.tkv_append(self._h, layer, self._dev_tensor(k, (B, n_new, Hkv, D)),
                                        self._dev_tensor(v, (B, n_new, Hkv, D)), n_new, self._stream(stream)))

    def attend_and_score(self, layer, q, out=None, stream=None):
        L, B, Hq, Hkv, D = self.shape
        if out is None:
            out = torch.empty((B, Hq, D), dtype=self.out_torch_dtype, device=self.device)
        self._check(self.lib.tkv_attend_and_score(self._h, layer, self._dev_tensor(q, (B, Hq, D)),
                                                  self._dev_tensor(out, (B, Hq, D), self.out_torch_dtype),
                                                  self._stream(stream)))
        return out

    def attend_and_score_noalloc(self, layer, q, out, stream=None):
        """The variant that allocates nothing: `out` must be passed in."""
        L, B, Hq, Hkv, D = self.shape
        self._check(self.lib.tkv_attend_and_score_noalloc(self._h, layer, self._dev_tensor(q, (B, Hq, D)),
                                                          self._dev_tensor(out, (B, Hq, D), self.out_torch_dtype),
                                                          self._stream(stream)))
        return out

    def attend_and_score_chunk(self, layer, q, out=None, stream=None):
        L, B, Hq, Hkv, D = self.shape
        n_q = int(q.shape[1])
        if out is None:
            out = torch.empty((B, n_q, Hq, D), dtype=self.out_torch_dtype, device=self.device)
        self._check(self.lib.tkv_attend_and_score_chunk(self._h, layer, self._dev_tensor(q, (B, n_q, Hq, D)),
                                                        self._dev_tensor(out, (B, n_q, Hq, D), self.out_torch_dtype),
                                                        n_q, self._stream(stream)))
        return out

    def decode_step(self, k_all, v_all, q_all, out_all=None, stream=None):
        L, B, Hq, Hkv, D = self.shape
        if out_all is None:
            out_all = torch.empty((L, B, Hq, D), dtype=self.out_torch_dtype, device=self.device)
        self._check(self.lib.tkv_decode_step(self._h, self._dev_tensor(k_all, (L, B, 1, Hkv, D)),
                                             self._dev_tensor(v_all, (L, B, 1, Hkv, D)),
                                             self._dev_tensor(q_all, (L, B, Hq, D)),
                                             self._dev_tensor(out_all, (L, B, Hq, D), self.out_torch_dtype),
                                             self._stream(stream)))
        return out_all

    def set_profile(self, on):
        self._check(self.lib.tkv_set_profile(self._h, int(on)))

    def classify(self, policy_ppm, stream=None, count_rule=0):
        pol = tkv_policy(*[int(x) for x in policy_ppm], int(count_rule))
        self._check(self.lib.tkv_classify(self._h, C.byref(pol), self._stream(stream)))

    def migrate(self, stream=None):
        self._check(self.lib.tkv_migrate(self._h, self._stream(stream)))

    # -- inspection --------------------------------------------------------------------------------
    def get_scores(self):
        out = np.empty((self.shape[1], self.max_tokens), np.float32)
        self._check(self.lib.tkv_get_scores(self._h, out.ctypes.data_as(C.c_void_p)))
        return out

    def set_scores(self, s):
        s = np.ascontiguousarray(s, np.float32)
        assert s.shape == (self.shape[1], self.max_tokens)
        self._check(self.lib.tkv_set_scores(self._h, s.ctypes.data_as(C.c_void_p)))

    def get_tiers(self):
        out = np.empty((self.shape[1], self.max_tokens), np.uint8)
        self._check(self.lib.tkv_get_tiers(self._h, out.ctypes.data_as(C.c_void_p)))
        return out

    def get_pending_tiers(self):
        out = np.empty((self.shape[1], self.max_tokens), np.uint8)
        self._check(self.lib.tkv_get_pending_tiers(self._h, out.ctypes.data_as(C.c_void_p)))
        return out

    def set_tiers(self, t):
        full = np.zeros((self.shape[1], self.max_tokens), np.uint8)
        t = np.asarray(t, np.uint8)
        full[:, :t.shape[1]] = t
        self._check(self.lib.tkv_set_tiers(self._h, full.ctypes.data_as(C.c_void_p)))

    def get_index_list(self, tier, seq):
        out = np.empty(self.max_tokens, np.int32)
        n = C.c_int32(0)
        self._check(self.lib.tkv_get_index_list(self._h, tier, seq, out.ctypes.data_as(C.c_void_p), C.byref(n)))
        return out[:n.value].copy()

    def get_t2_row(self, layer, seq, kv_head, pos, which):
        D = self.shape[4]
        if self.t2_format == "int8_row":
            codes, scales = np.empty(D, np.int8), np.empty(1, np.float32)
        else:
            codes, scales = np.empty(D // 2, np.uint8), np.empty(D // 32, np.uint16)
        self._check(self.lib.tkv_get_t2_row(self._h, layer, seq, kv_head, pos, which,
                                            codes.ctypes.data_as(C.c_void_p), scales.ctypes.data_as(C.c_void_p)))
        return codes, scales

    def get_row(self, layer, seq, kv_head, pos, which):
        D = self.shape[4]
        out = np.empty(D, np.float32 if self.kv_dtype == "f32" else np.uint16)
        self._check(self.lib.tkv_get_row(self._h, layer, seq, kv_head, pos, which, out.ctypes.data_as(C.c_void_p)))
        return out

    def wait_prefetch(self):
        self._check(self.lib.tkv_wait_prefetch(self._h))

    def get_stats(self):
        st = tkv_stats()
        self._check(self.lib.tkv_get_stats(self._h, C.byref(st)))
        return {name: (list(getattr(st, name)) if name == "tier_count" else getattr(st, name)) for name, _ in tkv_stats._fields_}

    def layer_length(self, layer):
        return int(self.lib.tkv_layer_length(self._h, layer))
