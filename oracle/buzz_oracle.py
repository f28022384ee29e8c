"""ctypes wrapper around ``buzz_oracle.c`` -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may
import this module.  It shares nothing with the HIP library and must never be
imported by it.  All arrays are float64 numpy arrays; inputs that were rounded
to fp16/bf16 for the GPU are widened exactly before they get here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "buzz_oracle.c")
_LIB = os.path.join(_HERE, "libbuzz_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent units only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("sink", ctypes.c_int32), ("window", ctypes.c_int32),
        ("segment", ctypes.c_int32), ("keep", ctypes.c_int32),
        ("evict_every", ctypes.c_int32), ("old_stride", ctypes.c_int32),
        ("auto_evict", ctypes.c_int32), ("variant", ctypes.c_int32),
        ("capacity", ctypes.c_int64), ("softmax_scale", ctypes.c_double),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.c_void_p
        lib.oracle_create.argtypes = [ctypes.POINTER(_Cfg), ctypes.POINTER(P)]
        lib.oracle_destroy.argtypes = [P]
        lib.oracle_destroy.restype = None
        lib.oracle_evict.argtypes = [P]
        lib.oracle_prefill.argtypes = [P, P, P, ctypes.c_int64, P, ctypes.c_int64, P]
        lib.oracle_decode_step.argtypes = [P, P, P, P, P]
        lib.oracle_len.argtypes = [P, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(ctypes.c_int64)]
        lib.oracle_export.argtypes = [P, P, P, P, P]
        lib.oracle_set_scores.argtypes = [P, P]
        _lib = lib
    return _lib


class OracleError(RuntimeError):
    pass


def _chk(rc: int, what: str):
    if rc != 0:
        raise OracleError(f"{what} failed with code {rc}")


def _f64(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


@dataclass
class OracleConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    sink: int
    window: int
    segment: int
    keep: int = 1
    evict_every: int = 1
    old_stride: int = 0       # 0 => floor((s+1)/2), the paper's default
    auto_evict: bool = True
    capacity: int = 0
    softmax_scale: float = 0.0
    log_n: bool = False            # Sec. 3.5: scale *= log(n)/log(512)
    threshold_total: bool = False  # T bounds old + new tokens (theorem proof's reading)
    interval_new: bool = False     # ablation (Sec. 4.3): new tokens interval-sampled, scores unused
    global_topk: bool = False      # H2O-style baseline (Sec. 4.1): top `keep` of all rows between sink and window


class OracleCache:
    """One BUZZ cache (one layer) held on the host in float64."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        self._lib = _load()
        c = _Cfg(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.sink, cfg.window,
                 cfg.segment, cfg.keep, cfg.evict_every, cfg.old_stride, int(cfg.auto_evict),
                 int(cfg.log_n) | (int(cfg.threshold_total) << 1) | (int(cfg.interval_new) << 2)
                 | (int(cfg.global_topk) << 3),
                 cfg.capacity, cfg.softmax_scale)
        h = ctypes.c_void_p()
        _chk(self._lib.oracle_create(ctypes.byref(c), ctypes.byref(h)), "oracle_create")
        self._h = h

    def __del__(self):
        h = getattr(self, "_h", None)
        if h:
            self._lib.oracle_destroy(h)
            self._h = None

    @property
    def units(self) -> int:
        return self.cfg.batch * self.cfg.n_kv_heads

    def prefill(self, K, V, q_obs=None, init_score=None):
        c = self.cfg
        K = _f64(K)
        N = K.shape[2]
        K = _f64(K, (c.batch, c.n_kv_heads, N, c.head_dim))
        V = _f64(V, (c.batch, c.n_kv_heads, N, c.head_dim))
        n_obs = 0
        qp = None
        if q_obs is not None and q_obs.shape[2] > 0:
            n_obs = q_obs.shape[2]
            q_obs = _f64(q_obs, (c.batch, c.n_q_heads, n_obs, c.head_dim))
            qp = q_obs.ctypes.data
        ip = None
        if init_score is not None:
            init_score = _f64(init_score, (c.batch, c.n_kv_heads, N))
            ip = init_score.ctypes.data
        _chk(self._lib.oracle_prefill(self._h, K.ctypes.data, V.ctypes.data, N, qp, n_obs, ip), "oracle_prefill")

    def decode_step(self, q, k_new, v_new):
        c = self.cfg
        q = _f64(q, (c.batch, c.n_q_heads, c.head_dim))
        k_new = _f64(k_new, (c.batch, c.n_kv_heads, c.head_dim))
        v_new = _f64(v_new, (c.batch, c.n_kv_heads, c.head_dim))
        out = np.empty((c.batch, c.n_q_heads, c.head_dim), dtype=np.float64)
        _chk(self._lib.oracle_decode_step(self._h, q.ctypes.data, k_new.ctypes.data, v_new.ctypes.data,
                                          out.ctypes.data), "oracle_decode_step")
        return out

    def evict(self):
        _chk(self._lib.oracle_evict(self._h), "oracle_evict")

    def lengths(self):
        n, n_old, nc = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        _chk(self._lib.oracle_len(self._h, ctypes.byref(n), ctypes.byref(n_old), ctypes.byref(nc)), "oracle_len")
        return n.value, n_old.value, nc.value

    def export(self):
        """Return (K, V, score, pos) of the retained rows in cache order."""
        c = self.cfg
        n, _, _ = self.lengths()
        K = np.empty((c.batch, c.n_kv_heads, n, c.head_dim), dtype=np.float64)
        V = np.empty_like(K)
        A = np.empty((c.batch, c.n_kv_heads, n), dtype=np.float64)
        pos = np.empty((c.batch, c.n_kv_heads, n), dtype=np.int32)
        _chk(self._lib.oracle_export(self._h, K.ctypes.data, V.ctypes.data, A.ctypes.data, pos.ctypes.data),
             "oracle_export")
        return K, V, A, pos

    def set_scores(self, A):
        c = self.cfg
        n, _, _ = self.lengths()
        A = _f64(A, (c.batch, c.n_kv_heads, n))
        _chk(self._lib.oracle_set_scores(self._h, A.ctypes.data), "oracle_set_scores")
