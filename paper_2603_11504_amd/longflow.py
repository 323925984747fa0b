"""Thin ctypes binding over ``liblongflow.so`` -- argument marshalling only.

Same names as the C ABI (include/longflow.h).  PyTorch supplies device memory and the
stream; every step of the decode path runs in the library's HIP kernels.  There is no
fallback: if the library has not been built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblongflow.so")

LF_OK, LF_ERR_INVALID_ARG, LF_ERR_UNSUPPORTED, LF_ERR_WORKSPACE, LF_ERR_STATE, LF_ERR_HIP = range(6)
LF_F32, LF_BF16 = 0, 1
LF_FLAG_ATTENTION_ONLY = 1
LF_FLAG_FORCE_VALU = 2
LF_FLAG_FORCE_SPLIT = 4
LF_FLAG_FORCE_UNIT = 8
LF_FLAG_UNFUSED_ACCUM = 16
LF_FLAG_MAX_FREE = 32
LF_EVICT_STATIC_MAX_SLOTS = 1 << 20

EXPORTS = ("longflow_workspace_bytes", "longflow_workspace_regions", "longflow_init_cache", "longflow_decode_step",
           "longflow_fill_steps", "longflow_compress_scratch_bytes", "longflow_compress_prompt", "longflow_scores", "longflow_set_pending", "longflow_set_mask", "longflow_get_mask", "longflow_evict_scratch_bytes",
           "longflow_evict_lowest", "longflow_evict_lowest_static", "longflow_valid_count",
           "longflow_destroy_cache", "longflow_last_error", "longflow_profile_begin",
           "longflow_profile_end", "longflow_plan_info", "longflow_group_workspace_bytes", "longflow_group_create",
           "longflow_group_decode_step", "longflow_group_destroy")


class lf_config(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("q_heads", ctypes.c_int32), ("kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("budget", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class lf_plan_info(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("workgroups_per_unit", ctypes.c_int32),
                ("slots_per_workgroup", ctypes.c_int32), ("launches_per_step", ctypes.c_int32),
                ("threads_per_workgroup", ctypes.c_int32), ("lds_bytes", ctypes.c_uint32)]


class lf_region(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 24), ("offset", ctypes.c_uint64), ("bytes", ctypes.c_uint64)]


LF_PATH_SPLIT_VALU, LF_PATH_SPLIT_MFMA, LF_PATH_UNIT_MFMA, LF_PATH_SPLIT_MFMA_F32 = range(4)
PATH_KERNELS = ("split_valu_kernel", "split_mfma_kernel", "unit_mfma_kernel", "split_mfma32_kernel")


class LongFlowError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"longflow status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """The loaded C library; raises if it was never built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.longflow_workspace_bytes.argtypes = [ctypes.POINTER(lf_config)]
        L.longflow_workspace_bytes.restype = ctypes.c_size_t
        L.longflow_workspace_regions.argtypes = [ctypes.POINTER(lf_config), ctypes.POINTER(lf_region), i32,
                                                 ctypes.POINTER(i32)]
        L.longflow_workspace_regions.restype = ctypes.c_int
        L.longflow_init_cache.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(lf_config), vp, vp, vp, vp,
                                          i32, vp, ctypes.c_size_t, vp]
        L.longflow_init_cache.restype = ctypes.c_int
        L.longflow_decode_step.argtypes = [vp] * 7
        L.longflow_decode_step.restype = ctypes.c_int
        L.longflow_fill_steps.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.longflow_fill_steps.restype = ctypes.c_int
        L.longflow_compress_scratch_bytes.argtypes = [ctypes.POINTER(lf_config), i32, i32]
        L.longflow_compress_scratch_bytes.restype = ctypes.c_size_t
        L.longflow_compress_prompt.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, vp]
        L.longflow_compress_prompt.restype = ctypes.c_int
        L.longflow_scores.argtypes = [vp, vp, vp]
        L.longflow_scores.restype = ctypes.c_int
        L.longflow_set_pending.argtypes = [vp, vp, vp]
        L.longflow_set_pending.restype = ctypes.c_int
        L.longflow_set_mask.argtypes = [vp, vp, vp]
        L.longflow_set_mask.restype = ctypes.c_int
        L.longflow_get_mask.argtypes = [vp, vp, vp]
        L.longflow_get_mask.restype = ctypes.c_int
        L.longflow_evict_scratch_bytes.argtypes = [ctypes.POINTER(lf_config)]
        L.longflow_evict_scratch_bytes.restype = ctypes.c_size_t
        L.longflow_evict_lowest.argtypes = [vp, i32, vp, ctypes.c_size_t, vp, vp]
        L.longflow_evict_lowest.restype = ctypes.c_int
        L.longflow_evict_lowest_static.argtypes = [vp, i32, vp, vp]
        L.longflow_evict_lowest_static.restype = ctypes.c_int
        L.longflow_valid_count.argtypes = [vp]
        L.longflow_valid_count.restype = ctypes.c_int
        L.longflow_destroy_cache.argtypes = [vp]
        L.longflow_destroy_cache.restype = ctypes.c_int
        L.longflow_profile_begin.argtypes = [vp, i32]
        L.longflow_profile_begin.restype = ctypes.c_int
        L.longflow_profile_end.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        L.longflow_profile_end.restype = ctypes.c_int
        L.longflow_plan_info.argtypes = [ctypes.POINTER(lf_config), ctypes.POINTER(lf_plan_info)]
        L.longflow_plan_info.restype = ctypes.c_int
        L.longflow_group_workspace_bytes.argtypes = [i32]
        L.longflow_group_workspace_bytes.restype = ctypes.c_size_t
        L.longflow_group_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), i32, vp, ctypes.c_size_t, vp]
        L.longflow_group_create.restype = ctypes.c_int
        L.longflow_group_decode_step.argtypes = [vp] * 7
        L.longflow_group_decode_step.restype = ctypes.c_int
        L.longflow_group_destroy.argtypes = [vp]
        L.longflow_group_destroy.restype = ctypes.c_int
        L.longflow_last_error.argtypes = []
        L.longflow_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != LF_OK:
        raise LongFlowError(rc, lib().longflow_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _arg(t, numel, dtype, what):
    """Device pointer of a tensor argument after checking what the C side cannot see: that it is a
    contiguous device tensor of the element type and count the kernels will read or write."""
    if t is None:
        return None
    if t.dtype is not dtype or t.numel() != numel or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{what}: need a contiguous device tensor of {numel} {dtype} elements, got "
                         f"{tuple(t.shape)} {t.dtype} on {t.device}{'' if t.is_contiguous() else ', not contiguous'}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_config(batch, q_heads, kv_heads, head_dim, budget, dtype, flags=0) -> lf_config:
    code = {torch.float32: LF_F32, torch.bfloat16: LF_BF16, "f32": LF_F32, "bf16": LF_BF16}[dtype]
    return lf_config(batch, q_heads, kv_heads, head_dim, budget, code, flags)


def longflow_workspace_bytes(cfg: lf_config) -> int:
    return int(lib().longflow_workspace_bytes(ctypes.byref(cfg)))


def longflow_workspace_regions(cfg: lf_config):
    """-> [(name, offset, bytes)] in address order: how the workspace is carved."""
    n = ctypes.c_int32()
    _check(lib().longflow_workspace_regions(ctypes.byref(cfg), None, 0, ctypes.byref(n)))
    regs = (lf_region * n.value)()
    _check(lib().longflow_workspace_regions(ctypes.byref(cfg), regs, n.value, ctypes.byref(n)))
    return [(r.name.decode(), int(r.offset), int(r.bytes)) for r in regs]


def longflow_plan_info(cfg: lf_config) -> lf_plan_info:
    info = lf_plan_info()
    _check(lib().longflow_plan_info(ctypes.byref(cfg), ctypes.byref(info)))
    return info


class LongFlowCache:
    """Owns the torch tensors behind one layer's static cache and its C handle."""

    def __init__(self, batch, q_heads, kv_heads, head_dim, budget, dtype=torch.bfloat16, flags=0,
                 device="cuda", k_init=None, v_init=None, k_cache=None, v_cache=None):
        self.cfg = make_config(batch, q_heads, kv_heads, head_dim, budget, dtype, flags)
        self.dtype = dtype
        self.device = torch.device(device)
        nbytes = longflow_workspace_bytes(self.cfg)
        if nbytes == 0:
            raise LongFlowError(LF_ERR_UNSUPPORTED, lib().longflow_last_error().decode())
        shape = (batch, kv_heads, budget, head_dim)
        # empty slots are never read: poison them so that a stray read shows up
        self.k_cache = k_cache if k_cache is not None else torch.full(shape, float("nan"), dtype=dtype, device=self.device)
        self.v_cache = v_cache if v_cache is not None else torch.full(shape, float("nan"), dtype=dtype, device=self.device)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        n_init = 0 if k_init is None else int(k_init.shape[2])
        if k_init is not None:
            k_init = k_init.contiguous()
            v_init = v_init.contiguous()
        h = ctypes.c_void_p()
        n_cache = batch * kv_heads * budget * head_dim
        n_rows = batch * kv_heads * n_init * head_dim
        _check(lib().longflow_init_cache(ctypes.byref(h), ctypes.byref(self.cfg), _arg(self.k_cache, n_cache, dtype, "k_cache"),
                                         _arg(self.v_cache, n_cache, dtype, "v_cache"), _arg(k_init, n_rows, dtype, "k_init"),
                                         _arg(v_init, n_rows, dtype, "v_init"), n_init,
                                         _ptr(self.workspace), nbytes, _stream()))
        self._h = h
        self.out = torch.empty((batch, q_heads, head_dim), dtype=dtype, device=self.device)
        self.evict_idx = torch.empty((batch, kv_heads), dtype=torch.int32, device=self.device)
        self._nq, self._nkv, self._nu = batch * q_heads * head_dim, batch * kv_heads * head_dim, batch * kv_heads

    def decode_step(self, q, k_new=None, v_new=None, out=None, evict_idx=None):
        """Asynchronous; returns (out, evict_idx) tensors owned by this object unless given."""
        out = self.out if out is None else out
        evict_idx = self.evict_idx if evict_idx is None else evict_idx
        dt = self.dtype
        _check(lib().longflow_decode_step(self._h, _arg(q, self._nq, dt, "q"), _arg(k_new, self._nkv, dt, "k_new"),
                                          _arg(v_new, self._nkv, dt, "v_new"), _arg(out, self._nq, dt, "out"),
                                          _arg(evict_idx, self._nu, torch.int32, "evict_idx"), _stream()))
        return out, evict_idx

    def fill_steps(self, q, k_new, v_new, out=None, evict_idx=None):
        """The next T tokens in one call (= T decode steps; those that find a free slot go in bulk):
        q [T,B,Hq,D], k_new, v_new [T,B,Hkv,D] (contiguous) -> (out [T,B,Hq,D], evict_idx [B,Hkv]
        as after the last of them)."""
        T = int(q.shape[0])
        if out is None:
            out = torch.empty((T, self.cfg.batch, self.cfg.q_heads, self.cfg.head_dim), dtype=self.dtype, device=self.device)
        evict_idx = self.evict_idx if evict_idx is None else evict_idx
        dt = self.dtype
        _check(lib().longflow_fill_steps(self._h, T, _arg(q, T * self._nq, dt, "q"), _arg(k_new, T * self._nkv, dt, "k_new"),
                                         _arg(v_new, T * self._nkv, dt, "v_new"), _arg(out, T * self._nq, dt, "out"),
                                         _arg(evict_idx, self._nu, torch.int32, "evict_idx"), _stream()))
        return out, evict_idx

    def compress_prompt(self, q_window, k_prompt, v_prompt, keep, pool=1, want_pooled=True):
        """A prompt longer than the budget into an empty cache: q_window [W,B,Hq,D], k_prompt, v_prompt
        [B,Hkv,T,D] (contiguous) -> (pooled votes [B,Hkv,T-W] float32 or None, kept rows [B,Hkv,keep] int32)."""
        W, T = int(q_window.shape[0]), int(k_prompt.shape[2])
        cfg, dt = self.cfg, self.dtype
        nbytes = int(lib().longflow_compress_scratch_bytes(ctypes.byref(cfg), T, W))
        scratch = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=self.device)
        pooled = torch.empty((cfg.batch, cfg.kv_heads, T - W), dtype=torch.float32, device=self.device) if want_pooled else None
        kept = torch.empty((cfg.batch, cfg.kv_heads, keep), dtype=torch.int32, device=self.device)
        _check(lib().longflow_compress_prompt(self._h, T, W, int(keep), int(pool), _arg(q_window, W * self._nq, dt, "q_window"),
                                              _arg(k_prompt, self._nu * T * cfg.head_dim, dt, "k_prompt"),
                                              _arg(v_prompt, self._nu * T * cfg.head_dim, dt, "v_prompt"),
                                              _ptr(scratch), nbytes, _ptr(pooled), _ptr(kept), _stream()))
        self._keep_scratch = scratch  # alive until the kernels that use it have run
        return pooled, kept

    def scores(self):
        s = torch.empty((self.cfg.batch, self.cfg.kv_heads, self.cfg.budget), dtype=torch.float32,
                        device=self.device)
        _check(lib().longflow_scores(self._h, _ptr(s), _stream()))
        return s

    def set_pending(self, slots):
        slots = slots.to(device=self.device, dtype=torch.int32).contiguous()
        _check(lib().longflow_set_pending(self._h, _ptr(slots), _stream()))
        self._keep = slots  # alive until the async copy has run

    def set_mask(self, mask):
        """mask: [B, Hkv, N], nonzero = valid slot (the vector M of Alg. 1)."""
        mask = (mask != 0).to(device=self.device, dtype=torch.uint8).contiguous()
        assert tuple(mask.shape) == (self.cfg.batch, self.cfg.kv_heads, self.cfg.budget)
        _check(lib().longflow_set_mask(self._h, _ptr(mask), _stream()))
        self._keep_mask = mask  # alive until the kernels that read it have run

    def mask(self):
        """-> uint8 [B, Hkv, N], 1 where the slot holds a token."""
        m = torch.empty((self.cfg.batch, self.cfg.kv_heads, self.cfg.budget), dtype=torch.uint8, device=self.device)
        _check(lib().longflow_get_mask(self._h, _ptr(m), _stream()))
        return m

    def evict_lowest(self, k):
        """Drop the k lowest-scoring valid slots per (batch, KV head) -> their slots [B, Hkv, k] int32."""
        nbytes = int(lib().longflow_evict_scratch_bytes(ctypes.byref(self.cfg)))
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        ev = torch.empty((self.cfg.batch, self.cfg.kv_heads, k), dtype=torch.int32, device=self.device)
        _check(lib().longflow_evict_lowest(self._h, k, _ptr(scratch), nbytes, _ptr(ev), _stream()))
        self._keep_scratch = scratch  # alive until the kernels that use it have run
        return ev

    def evict_lowest_static(self, k, evicted=None):
        """evict_lowest through the library's built-in scratch (no scratch buffer is passed or
        allocated); `evicted` [B, Hkv, k] int32 may be given so that the call allocates nothing at all."""
        if evicted is None:
            evicted = torch.empty((self.cfg.batch, self.cfg.kv_heads, k), dtype=torch.int32, device=self.device)
        _check(lib().longflow_evict_lowest_static(self._h, k, _arg(evicted, self._nu * k, torch.int32, "evicted"), _stream()))
        return evicted

    def profile_begin(self, max_steps):
        _check(lib().longflow_profile_begin(self._h, max_steps))

    def profile_end(self):
        """-> (kernel milliseconds summed over the recorded steps, number of steps)."""
        ms = ctypes.c_float()
        n = ctypes.c_int32()
        _check(lib().longflow_profile_end(self._h, ctypes.byref(ms), ctypes.byref(n)))
        return float(ms.value), int(n.value)

    @property
    def valid_count(self):
        return int(lib().longflow_valid_count(self._h))

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib().longflow_destroy_cache(self._h)
            self._h = None

    def __del__(self):
        try:
            if getattr(self, "_h", None):
                lib().longflow_destroy_cache(self._h)
                self._h = None
        except Exception:
            pass


class LongFlowGroup:
    """Caches of one configuration and fill level that take their decode step in one launch."""

    def __init__(self, caches):
        self.caches = list(caches)
        n = len(self.caches)
        c0 = self.caches[0]
        self.device = c0.device
        nbytes = int(lib().longflow_group_workspace_bytes(n))
        self.workspace = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=self.device)
        handles = (ctypes.c_void_p * n)(*[c._h for c in self.caches])
        h = ctypes.c_void_p()
        _check(lib().longflow_group_create(ctypes.byref(h), handles, n, _ptr(self.workspace), nbytes, _stream()))
        self._h = h
        cfg = c0.cfg
        self.out = torch.empty((n, cfg.batch, cfg.q_heads, cfg.head_dim), dtype=c0.dtype, device=self.device)
        self.evict_idx = torch.empty((n, cfg.batch, cfg.kv_heads), dtype=torch.int32, device=self.device)

    def decode_step(self, q, k_new=None, v_new=None, out=None, evict_idx=None):
        """q/out: [n_caches, B, Hq, D]; k_new/v_new: [n_caches, B, Hkv, D], all contiguous."""
        out = self.out if out is None else out
        evict_idx = self.evict_idx if evict_idx is None else evict_idx
        c0, n = self.caches[0], len(self.caches)
        dt = c0.dtype
        _check(lib().longflow_group_decode_step(self._h, _arg(q, n * c0._nq, dt, "q"), _arg(k_new, n * c0._nkv, dt, "k_new"),
                                                _arg(v_new, n * c0._nkv, dt, "v_new"), _arg(out, n * c0._nq, dt, "out"),
                                                _arg(evict_idx, n * c0._nu, torch.int32, "evict_idx"), _stream()))
        return out, evict_idx

    def close(self):
        if getattr(self, "_h", None):
            torch.cuda.synchronize(self.device)
            lib().longflow_group_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            if getattr(self, "_h", None):
                lib().longflow_group_destroy(self._h)
                self._h = None
        except Exception:
            pass
