"""ctypes binding of the C ABI declared in ``include/buzz.h``.

Argument marshalling only: every step of the decode path runs in the HIP kernels of ``libbuzz.so``.
PyTorch supplies device memory (tensors' ``data_ptr()``) and the HIP stream; nothing here computes.
There is no fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libbuzz.so")

FLAG_AUTO_EVICT = 1
FLAG_DRY_RUN = 2
FLAG_STREAMING = 4
FLAG_CACHED = 8
FLAG_LOG_N = 16
FLAG_THRESHOLD_TOTAL = 32
FLAG_DETERMINISTIC = 64
FLAG_INTERVAL_NEW = 128
FLAG_DEVICE_MERGE = 256
FLAG_GLOBAL_TOPK = 512
DTYPE_CODES = {"fp32": 0, "fp16": 1, "bf16": 2}

EXPORTS = ["buzz_workspace_bytes", "buzz_cache_create", "buzz_prefill", "buzz_decode_step",
           "buzz_decode_step_static", "buzz_evict",
           "buzz_cache_destroy", "buzz_cache_len", "buzz_cache_export", "buzz_cache_import", "buzz_cache_set_splits",
           "buzz_cache_override_die_map", "buzz_cache_profile",
           "buzz_cache_profile_read", "buzz_bench_copy", "buzz_suggest_threshold", "buzz_strerror"]


class BuzzError(RuntimeError):
    def __init__(self, code: int, what: str, text: str):
        super().__init__(f"{what}: {text} ({code})")
        self.code = code


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("sink", ctypes.c_int32),
        ("window", ctypes.c_int32), ("segment", ctypes.c_int32), ("keep", ctypes.c_int32),
        ("evict_every", ctypes.c_int32), ("old_stride", ctypes.c_int32), ("flags", ctypes.c_uint32),
        ("max_context", ctypes.c_int64), ("capacity", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float), ("reserved", ctypes.c_int32),
    ]


class _Profile(ctypes.Structure):
    _fields_ = [("attn_launches", ctypes.c_int64), ("epilogue_launches", ctypes.c_int64),
                ("evictions", ctypes.c_int64), ("attn_ms", ctypes.c_double), ("epilogue_ms", ctypes.c_double),
                ("evict_ms", ctypes.c_double), ("attn_row_bytes", ctypes.c_double)]


@dataclass
class BuzzConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str          # "fp32" | "fp16" | "bf16"
    sink: int
    window: int
    segment: int
    keep: int
    evict_every: int
    max_context: int
    old_stride: int = 0    # 0 => floor((s+1)/2), the paper's default; 1 => survivors persist
    flags: int = FLAG_AUTO_EVICT
    capacity: int = 0
    softmax_scale: float = 0.0

    def to_c(self) -> _Cfg:
        return _Cfg(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, DTYPE_CODES[self.kv_dtype],
                    self.sink, self.window, self.segment, self.keep, self.evict_every, self.old_stride,
                    self.flags, self.max_context, self.capacity, self.softmax_scale, 0)


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load ``libbuzz.so``; build it first if it has never been built.  Raises if that fails."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    P, I64 = ctypes.c_void_p, ctypes.c_int64
    lib.buzz_workspace_bytes.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(ctypes.c_size_t)]
    lib.buzz_cache_create.argtypes = [ctypes.POINTER(_Cfg), P, ctypes.c_size_t, ctypes.POINTER(P)]
    lib.buzz_prefill.argtypes = [P, P, P, I64, P, I64, P, P]
    lib.buzz_decode_step.argtypes = [P, P, P, P, P, P]
    lib.buzz_decode_step_static.argtypes = [P, P, P, P, P, P]
    lib.buzz_evict.argtypes = [P, P]
    lib.buzz_cache_destroy.argtypes = [P]
    lib.buzz_cache_len.argtypes = [P, ctypes.POINTER(I64), ctypes.POINTER(I64), ctypes.POINTER(I64)]
    lib.buzz_cache_export.argtypes = [P, P, P, P, P, P]
    lib.buzz_cache_import.argtypes = [P, P, P, P, P, I64, I64, I64, P]
    lib.buzz_cache_set_splits.argtypes = [P, ctypes.c_int32]
    lib.buzz_cache_override_die_map.argtypes = [P, I64]
    lib.buzz_cache_profile.argtypes = [P, ctypes.c_int]
    lib.buzz_cache_profile_read.argtypes = [P, ctypes.POINTER(_Profile)]
    lib.buzz_bench_copy.argtypes = [P, P, ctypes.c_size_t, P]
    lib.buzz_suggest_threshold.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.buzz_suggest_threshold.restype = ctypes.c_int64
    lib.buzz_strerror.argtypes = [ctypes.c_int]
    lib.buzz_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise BuzzError(rc, what, load_library().buzz_strerror(rc).decode())


def workspace_bytes(cfg: BuzzConfig) -> int:
    out = ctypes.c_size_t()
    c = cfg.to_c()
    _check(load_library().buzz_workspace_bytes(ctypes.byref(c), ctypes.byref(out)), "buzz_workspace_bytes")
    return out.value


def suggest_threshold(segment: int, window: int) -> int:
    """Eviction threshold recommended by the Parameter Estimation theorem (Sec. 3.4) for FLAG_THRESHOLD_TOTAL."""
    return load_library().buzz_suggest_threshold(segment, window)


def bench_copy(dst, src, stream=None):
    """Plain device copy of ``src`` into ``dst`` (same byte size) with the library's own copy kernel."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().buzz_bench_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream)), "buzz_bench_copy")


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


class BuzzCache:
    """One layer's BUZZ cache on the GPU.  Tensors must be contiguous, on the GPU and of the config's dtype."""

    def __init__(self, cfg: BuzzConfig, device="cuda"):
        self.cfg = cfg
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.nbytes = workspace_bytes(cfg)
        self.dry = bool(cfg.flags & FLAG_DRY_RUN)
        self.workspace = None
        ws_ptr = None
        if not self.dry:
            import torch
            self.workspace = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
            ws_ptr = self.workspace.data_ptr()
        c = cfg.to_c()
        _check(self._lib.buzz_cache_create(ctypes.byref(c), ws_ptr, self.nbytes, ctypes.byref(self._h)),
               "buzz_cache_create")

    def close(self):
        if getattr(self, "_h", None):
            self._lib.buzz_cache_destroy(self._h)
            self._h = None

    __del__ = close

    def _stream(self, stream):
        return None if self.dry else _stream(stream)

    def prefill(self, k, v, q_obs=None, init_score=None, stream=None, n_prompt=None):
        n_prompt = k.shape[2] if n_prompt is None else n_prompt
        n_obs = 0 if q_obs is None else q_obs.shape[2]
        _check(self._lib.buzz_prefill(self._h, _ptr(k), _ptr(v), n_prompt, _ptr(q_obs) if n_obs else None, n_obs,
                                      _ptr(init_score), self._stream(stream)), "buzz_prefill")

    def decode_step(self, q, k_new, v_new, out, stream=None):
        _check(self._lib.buzz_decode_step(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                          self._stream(stream)), "buzz_decode_step")

    def decode_step_static(self, q, k_new, v_new, out, stream=None):
        """``decode_step`` with the split-softmax scratch in the library's static device array (allocates nothing)."""
        _check(self._lib.buzz_decode_step_static(self._h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out),
                                                 self._stream(stream)), "buzz_decode_step_static")

    def evict(self, stream=None):
        _check(self._lib.buzz_evict(self._h, self._stream(stream)), "buzz_evict")

    def lengths(self):
        n, n_old, nc = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _check(self._lib.buzz_cache_len(self._h, ctypes.byref(n), ctypes.byref(n_old), ctypes.byref(nc)),
               "buzz_cache_len")
        return n.value, n_old.value, nc.value

    def set_splits(self, n_splits: int):
        _check(self._lib.buzz_cache_set_splits(self._h, n_splits), "buzz_cache_set_splits")

    def override_die_map(self, die_map: int):
        _check(self._lib.buzz_cache_override_die_map(self._h, die_map), "buzz_cache_override_die_map")

    def profile(self, enable: bool):
        _check(self._lib.buzz_cache_profile(self._h, int(enable)), "buzz_cache_profile")

    def profile_read(self) -> dict:
        p = _Profile()
        _check(self._lib.buzz_cache_profile_read(self._h, ctypes.byref(p)), "buzz_cache_profile_read")
        return {k: getattr(p, k) for k, _ in _Profile._fields_}

    def import_rows(self, k, v, score, pos, n_old: int, tokens_seen: int, stream=None, n=None):
        """Load retained rows (as ``export`` returns them) into this cache; ``n`` only for dry-run caches."""
        n = k.shape[2] if n is None else n
        _check(self._lib.buzz_cache_import(self._h, _ptr(k), _ptr(v), _ptr(score), _ptr(pos), n, n_old, tokens_seen,
                                           self._stream(stream)), "buzz_cache_import")

    def export(self, stream=None):
        """Retained rows in cache order: (K, V, score, pos) as new GPU tensors."""
        import torch
        c = self.cfg
        n, _, _ = self.lengths()
        dt = {"fp32": torch.float32, "fp16": torch.float16, "bf16": torch.bfloat16}[c.kv_dtype]
        dev = self.workspace.device
        K = torch.empty(c.batch, c.n_kv_heads, n, c.head_dim, dtype=dt, device=dev)
        V = torch.empty_like(K)
        score = torch.empty(c.batch, c.n_kv_heads, n, dtype=torch.float32, device=dev)
        pos = torch.empty(c.batch, c.n_kv_heads, n, dtype=torch.int32, device=dev)
        _check(self._lib.buzz_cache_export(self._h, _ptr(K), _ptr(V), _ptr(score), _ptr(pos), self._stream(stream)),
               "buzz_cache_export")
        return K, V, score, pos
