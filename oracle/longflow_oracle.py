"""ctypes front-end of the float64 CPU oracle in ``longflow_oracle.c``.

Test infrastructure only: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; the GPU package never does.
Argument marshalling only -- every number comes out of the C file.

All arrays are float64, C-contiguous:
  q [B,Hq,D]; k_new, v_new [B,Hkv,D]; out [B,Hq,D]; scores [B,Hkv,N];
  evict_idx int32 [B,Hkv].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "longflow_oracle.c")
_LIB = os.path.join(_HERE, "liblongflow_oracle.so")
_LIB_SANITIZED = os.path.join(_HERE, "liblongflow_oracle_san.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent units).

    sanitize: the same file under AddressSanitizer + UndefinedBehaviorSanitizer (any report
    aborts), as a library of its own; the process that loads it must have libasan preloaded.
    """
    out = _LIB_SANITIZED if sanitize else _LIB
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=all"] if sanitize else ["-O2"]
        cmd = ["gcc", *opt, "-std=c11", "-fopenmp", "-fPIC", "-shared",
               "-fvisibility=hidden", "-o", out, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return out


_lib = None


def lib():
    global _lib
    if _lib is None:
        # LFO_SANITIZE=1: run everything through the sanitizer build (see tests/test_oracle_sanitized.py)
        L = ctypes.CDLL(build(sanitize=os.environ.get("LFO_SANITIZE") == "1"))
        L.lfo_attend_unit.argtypes = [ctypes.c_int] * 3 + [_dp] * 6
        L.lfo_attend_unit.restype = None
        L.lfo_argmin.argtypes = [ctypes.c_int, _dp]
        L.lfo_argmin.restype = ctypes.c_int
        L.lfo_cache_create.argtypes = [ctypes.c_int] * 5
        L.lfo_cache_create.restype = ctypes.c_void_p
        L.lfo_cache_destroy.argtypes = [ctypes.c_void_p]
        L.lfo_cache_destroy.restype = None
        L.lfo_cache_init.argtypes = [ctypes.c_void_p, _dp, _dp, ctypes.c_int]
        L.lfo_cache_init.restype = ctypes.c_int
        L.lfo_cache_step.argtypes = [ctypes.c_void_p, _dp, _dp, _dp, _dp, _ip]
        L.lfo_cache_step.restype = ctypes.c_int
        L.lfo_cache_fill.argtypes = [ctypes.c_void_p, ctypes.c_int, _dp, _dp, _dp, _dp, _ip]
        L.lfo_cache_fill.restype = ctypes.c_int
        L.lfo_cache_count.argtypes = [ctypes.c_void_p]
        L.lfo_cache_count.restype = ctypes.c_int
        L.lfo_cache_scores.argtypes = [ctypes.c_void_p, _dp]
        L.lfo_cache_scores.restype = None
        L.lfo_cache_get_pending.argtypes = [ctypes.c_void_p, _ip]
        L.lfo_cache_get_pending.restype = None
        L.lfo_cache_set_pending.argtypes = [ctypes.c_void_p, _ip]
        L.lfo_cache_set_pending.restype = ctypes.c_int
        L.lfo_cache_get_kv.argtypes = [ctypes.c_void_p, _dp, _dp]
        L.lfo_cache_get_kv.restype = None
        _bp = ctypes.POINTER(ctypes.c_uint8)
        L.lfo_cache_set_mask.argtypes = [ctypes.c_void_p, _bp]
        L.lfo_cache_set_mask.restype = ctypes.c_int
        L.lfo_cache_get_mask.argtypes = [ctypes.c_void_p, _bp]
        L.lfo_cache_get_mask.restype = ctypes.c_int
        L.lfo_cache_evict_lowest.argtypes = [ctypes.c_void_p, ctypes.c_int, _ip]
        L.lfo_cache_evict_lowest.restype = ctypes.c_int
        L.lfo_cache_set_rule.argtypes = [ctypes.c_void_p, ctypes.c_int]
        L.lfo_cache_set_rule.restype = ctypes.c_int
        L.lfo_compress_prompt.argtypes = [ctypes.c_int] * 8 + [_dp, _dp, _dp, _ip]
        L.lfo_compress_prompt.restype = ctypes.c_int
        L.lfo_num_threads.argtypes = []
        L.lfo_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _d(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a):
    return a.ctypes.data_as(_dp)


def attend_unit(q, K, V, want_alpha=False):
    """One KV head: q [G,D], K,V [n,D] -> (out [G,D], score [n], alpha [G,n]|None)."""
    q = _d(q); K = _d(K); V = _d(V)
    G, D = q.shape
    n = K.shape[0]
    assert K.shape == (n, D) and V.shape == (n, D) and n >= 1
    out = np.empty((G, D)); score = np.empty(n)
    alpha = np.empty((G, n)) if want_alpha else None
    lib().lfo_attend_unit(n, D, G, _ptr(q), _ptr(K), _ptr(V), _ptr(out),
                          _ptr(alpha) if want_alpha else None, _ptr(score))
    return out, score, alpha


def argmin(x):
    x = _d(x)
    return int(lib().lfo_argmin(x.size, _ptr(x)))


def compress_prompt(q_window, K, keep, pool=1):
    """A prompt longer than the budget, cut to `keep` rows by observation-window voting.
    q_window [W,B,Hq,D] (queries of the last W prompt positions), K [B,Hkv,T,D]
    -> (pooled votes [B,Hkv,T-W], kept positions [B,Hkv,keep] ascending)."""
    q_window = _d(q_window); K = _d(K)
    W, B, Hq, D = q_window.shape
    _, Hkv, T, _ = K.shape
    assert K.shape == (B, Hkv, T, D)
    pooled = np.empty((B, Hkv, T - W))
    kept = np.empty((B, Hkv, keep), dtype=np.int32)
    if lib().lfo_compress_prompt(B, Hq, Hkv, D, T, W, int(keep), int(pool), _ptr(q_window), _ptr(K),
                                 _ptr(pooled), kept.ctypes.data_as(_ip)):
        raise ValueError("need 1 <= W <= keep <= T and an odd pool width")
    return pooled, kept


def num_threads() -> int:
    return int(lib().lfo_num_threads())


class OracleCache:
    """Static fixed-budget KV cache advanced one decode step at a time."""

    RULES = {"longflow": 0, "accumulated_attention": 1}

    def __init__(self, batch, q_heads, kv_heads, head_dim, budget, rule="longflow"):
        self.B, self.Hq, self.Hkv, self.D, self.N = batch, q_heads, kv_heads, head_dim, budget
        self._h = lib().lfo_cache_create(batch, q_heads, kv_heads, head_dim, budget)
        if not self._h:
            raise ValueError("invalid oracle geometry")
        if lib().lfo_cache_set_rule(self._h, self.RULES[rule]):
            raise ValueError("importance rule refused")

    def __del__(self):
        try:
            if getattr(self, "_h", None):
                lib().lfo_cache_destroy(self._h)
                self._h = None
        except Exception:       # interpreter shutdown: module globals may already be gone
            pass

    def init(self, k_init=None, v_init=None):
        n_init = 0 if k_init is None else int(np.shape(k_init)[2])
        if n_init:
            k = _d(k_init, (self.B, self.Hkv, n_init, self.D))
            v = _d(v_init, (self.B, self.Hkv, n_init, self.D))
            rc = lib().lfo_cache_init(self._h, _ptr(k), _ptr(v), n_init)
        else:
            rc = lib().lfo_cache_init(self._h, None, None, 0)
        if rc:
            raise ValueError("n_init out of range")

    def step(self, q, k_new, v_new):
        """-> (out [B,Hq,D] float64, evict_idx [B,Hkv] int32)."""
        q = _d(q, (self.B, self.Hq, self.D))
        k = _d(k_new, (self.B, self.Hkv, self.D))
        v = _d(v_new, (self.B, self.Hkv, self.D))
        out = np.empty((self.B, self.Hq, self.D))
        idx = np.empty((self.B, self.Hkv), dtype=np.int32)
        rc = lib().lfo_cache_step(self._h, _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                  idx.ctypes.data_as(_ip))
        if rc:
            raise RuntimeError("cache is full and has no pending slot")
        return out, idx

    def fill(self, q, k_new, v_new):
        """The next T tokens in one call (T consecutive steps): q [T,B,Hq,D], k_new, v_new [T,B,Hkv,D]
        -> (out [T,B,Hq,D], evict_idx [B,Hkv] of the last token)."""
        T = int(np.shape(q)[0])
        q = _d(q, (T, self.B, self.Hq, self.D))
        k = _d(k_new, (T, self.B, self.Hkv, self.D))
        v = _d(v_new, (T, self.B, self.Hkv, self.D))
        out = np.empty((T, self.B, self.Hq, self.D))
        idx = np.empty((self.B, self.Hkv), dtype=np.int32)
        if lib().lfo_cache_fill(self._h, T, _ptr(q), _ptr(k), _ptr(v), _ptr(out), idx.ctypes.data_as(_ip)):
            raise ValueError("T < 1, or a full cache without a pending slot")
        return out, idx

    @property
    def count(self):
        return int(lib().lfo_cache_count(self._h))

    def scores(self):
        s = np.empty((self.B, self.Hkv, self.N))
        lib().lfo_cache_scores(self._h, _ptr(s))
        return s

    def pending(self):
        p = np.empty((self.B, self.Hkv), dtype=np.int32)
        lib().lfo_cache_get_pending(self._h, p.ctypes.data_as(_ip))
        return p

    def set_pending(self, slots):
        s = np.ascontiguousarray(slots, dtype=np.int32).reshape(self.B, self.Hkv)
        if lib().lfo_cache_set_pending(self._h, s.ctypes.data_as(_ip)):
            raise ValueError("pending slot out of range")

    def kv(self):
        shape = (self.B, self.Hkv, self.N, self.D)
        K = np.empty(shape); V = np.empty(shape)
        lib().lfo_cache_get_kv(self._h, _ptr(K), _ptr(V))
        return K, V

    def set_mask(self, mask):
        """Explicit validity mask [B,Hkv,N] (nonzero = valid); switches the cache to mask mode."""
        m = np.ascontiguousarray(np.asarray(mask) != 0, dtype=np.uint8).reshape(self.B, self.Hkv, self.N)
        if lib().lfo_cache_set_mask(self._h, m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))):
            raise ValueError("this importance rule takes no mask")

    def mask(self):
        m = np.empty((self.B, self.Hkv, self.N), dtype=np.uint8)
        lib().lfo_cache_get_mask(self._h, m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
        return m

    def evict_lowest(self, k):
        """Drop the k lowest-scoring valid slots of every unit at once -> their slots [B,Hkv,k]."""
        ev = np.empty((self.B, self.Hkv, k), dtype=np.int32)
        if lib().lfo_cache_evict_lowest(self._h, int(k), ev.ctypes.data_as(_ip)):
            raise ValueError("k out of range, or not available under this importance rule")
        return ev
