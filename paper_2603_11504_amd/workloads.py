"""Seeded synthetic decode workloads (inputs only -- none of the method's arithmetic).

Shared by the GPU path's tests/benchmark and by the CPU oracle's tests; this
module draws random numbers, applies the workload's input *structure* (sink
token, outlier channels, per-channel key scales), rounds once to the storage
dtype and hands the same bits to whoever asks.  It imports neither the GPU
binding nor the oracle.

The five workloads stand in for the paper's real-model decodes (Sec. 4.1:
GQA reasoning models, head_dim 128, budget = a fixed fraction of a long
output, one eviction per decode step); no benchmark item is reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20260311


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # storage dtype of q/K/V/out: "f32" or "bf16"
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    budget: int           # N: slots of the static cache
    n_init: int           # rows pre-filled before the first decode step
    steps: int            # decode steps of the run
    layers: int = 1       # independent caches advanced per step
    sink_scale: float = 1.0        # key of token 0 multiplied by this
    outlier_channels: int = 0      # this many key channels per KV head ...
    outlier_scale: float = 1.0     # ... multiplied by this
    channel_scale_range: Optional[Tuple[float, float]] = None  # keys * U(lo,hi) per (kv head, channel)
    seed: int = BASE_SEED

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def units(self) -> int:
        return self.batch * self.kv_heads

    def kv_bytes_per_call(self, n: Optional[int] = None) -> int:
        """Algorithmic bytes of one decode call: K and V rows of the valid slots, read once."""
        n = self.budget if n is None else n
        return 2 * self.units * n * self.head_dim * self.elem_bytes


# the benchmark spec `configs`, in order.
CONFIGS = (
    Workload("cfg0_f32_b1_4x1_d64_n256", "f32", 1, 4, 1, 64, 256, 0, 512,
             sink_scale=4.0, seed=BASE_SEED + 0),
    Workload("cfg1_bf16_b1_28x4_d128_n2048", "bf16", 1, 28, 4, 128, 2048, 0, 4096,
             outlier_channels=4, outlier_scale=8.0, seed=BASE_SEED + 1),
    Workload("cfg2_bf16_b32_28x4_d128_n4096", "bf16", 32, 28, 4, 128, 4096, 4095, 100,
             channel_scale_range=(0.5, 4.0), seed=BASE_SEED + 2),
    Workload("cfg3_bf16_b64_28x4_d128_n8192_l28", "bf16", 64, 28, 4, 128, 8192, 8191, 256,
             layers=28, sink_scale=4.0, seed=BASE_SEED + 3),
    Workload("cfg4_bf16_b128_40x8_d128_n16384", "bf16", 128, 40, 8, 128, 16384, 16383, 50,
             sink_scale=4.0, seed=BASE_SEED + 4),
)


def scaled(wl: Workload, **kw) -> Workload:
    """A smaller/larger variant of a workload with the same input structure."""
    return replace(wl, **kw)


# ---------------------------------------------------------------- bf16 bits

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 array holding exactly the values the storage dtype can represent."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    raise ValueError(dtype)


# ---------------------------------------------------------------- host (numpy) generators

def _rng(wl: Workload, stream: int, layer: int, t: int) -> np.random.Generator:
    # counter-based: any (stream, layer, step) can be drawn on its own
    return np.random.Generator(np.random.Philox(key=[wl.seed, (stream << 40) | (layer << 32) | t]))


def key_channel_scale(wl: Workload, layer: int = 0) -> np.ndarray:
    """float32 [Hkv, D] multiplier applied to every key (cached and new)."""
    s = np.ones((wl.kv_heads, wl.head_dim), dtype=np.float32)
    g = _rng(wl, 3, layer, 0)
    if wl.channel_scale_range is not None:
        lo, hi = wl.channel_scale_range
        s *= g.uniform(lo, hi, size=s.shape).astype(np.float32)
    if wl.outlier_channels:
        for h in range(wl.kv_heads):
            ch = g.choice(wl.head_dim, size=wl.outlier_channels, replace=False)
            s[h, ch] *= np.float32(wl.outlier_scale)
    return s


def host_prefill(wl: Workload, layer: int = 0):
    """K, V float32 [B,Hkv,n_init,D] (storage-rounded) for tokens 0..n_init-1, or (None, None)."""
    if wl.n_init == 0:
        return None, None
    g = _rng(wl, 1, layer, 0)
    shape = (wl.batch, wl.kv_heads, wl.n_init, wl.head_dim)
    k = g.standard_normal(shape, dtype=np.float32)
    v = g.standard_normal(shape, dtype=np.float32)
    k *= key_channel_scale(wl, layer)[None, :, None, :]
    k[:, :, 0, :] *= np.float32(wl.sink_scale)
    return round_to_storage(k, wl.dtype), round_to_storage(v, wl.dtype)


def host_step(wl: Workload, t: int, layer: int = 0):
    """q [B,Hq,D], k_new, v_new [B,Hkv,D] float32 (storage-rounded) of decode step t (0-based)."""
    g = _rng(wl, 2, layer, t)
    q = g.standard_normal((wl.batch, wl.q_heads, wl.head_dim), dtype=np.float32)
    k = g.standard_normal((wl.batch, wl.kv_heads, wl.head_dim), dtype=np.float32)
    v = g.standard_normal((wl.batch, wl.kv_heads, wl.head_dim), dtype=np.float32)
    k *= key_channel_scale(wl, layer)[None, :, :]
    if wl.n_init == 0 and t == 0:
        k *= np.float32(wl.sink_scale)      # token 0 arrives through the first decode step
    return (round_to_storage(q, wl.dtype), round_to_storage(k, wl.dtype),
            round_to_storage(v, wl.dtype))


# ---------------------------------------------------------------- device (torch) generators

def torch_dtype(wl: Workload):
    import torch
    return torch.float32 if wl.dtype == "f32" else torch.bfloat16


def to_torch(x: np.ndarray, wl: Workload, device):
    """Storage-rounded float32 numpy array -> torch tensor of the storage dtype (exact)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(device=device, dtype=torch_dtype(wl))


def to_f64(x) -> np.ndarray:
    """torch tensor (any float dtype, any device) or numpy array -> float64 numpy, exactly."""
    if isinstance(x, np.ndarray):
        return x.astype(np.float64)
    return x.detach().to("cpu").double().numpy()


def _torch_gen(wl: Workload, stream: int, layer: int, t: int, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(((wl.seed * 1000003 + stream * 7919 + layer) * 65537 + t) % (1 << 63))  # any seed fits
    return g


def device_prefill(wl: Workload, device, layer: int = 0):
    """K, V tensors [B,Hkv,n_init,D] in the storage dtype, drawn on `device`.

    For the large workloads, whose caches are too big to draw on the host.
    The values differ from host_prefill's (different generator); whoever checks
    against the oracle copies the rows it needs back from these tensors.
    """
    import torch
    if wl.n_init == 0:
        return None, None
    dt = torch_dtype(wl)
    shape = (wl.batch, wl.kv_heads, wl.n_init, wl.head_dim)
    g = _torch_gen(wl, 1, layer, 0, device)
    scale = torch.from_numpy(key_channel_scale(wl, layer)).to(device)[None, :, None, :]
    k = torch.empty(shape, dtype=dt, device=device)
    v = torch.empty(shape, dtype=dt, device=device)
    # one batch row at a time keeps the float32 temporaries small
    for b in range(wl.batch):
        kb = torch.randn(shape[1:], generator=g, device=device, dtype=torch.float32) * scale[0]
        kb[:, 0, :] *= wl.sink_scale
        k[b] = kb.to(dt)
        v[b] = torch.randn(shape[1:], generator=g, device=device, dtype=torch.float32).to(dt)
    return k, v


def device_step(wl: Workload, t: int, device, layer: int = 0):
    """q, k_new, v_new tensors of decode step t in the storage dtype, drawn on `device`."""
    import torch
    dt = torch_dtype(wl)
    g = _torch_gen(wl, 2, layer, t, device)
    scale = torch.from_numpy(key_channel_scale(wl, layer)).to(device)[None]
    q = torch.randn((wl.batch, wl.q_heads, wl.head_dim), generator=g, device=device, dtype=torch.float32)
    k = torch.randn((wl.batch, wl.kv_heads, wl.head_dim), generator=g, device=device, dtype=torch.float32) * scale
    v = torch.randn((wl.batch, wl.kv_heads, wl.head_dim), generator=g, device=device, dtype=torch.float32)
    if wl.n_init == 0 and t == 0:
        k = k * wl.sink_scale
    return q.to(dt), k.to(dt), v.to(dt)


def device_prompt(wl: Workload, T: int, W: int, device, layer: int = 0):
    """A prompt of T tokens in the workload's input structure, drawn on `device` in the storage
    dtype: (q_window [W,B,Hq,D], the queries of the last W tokens; K, V [B,Hkv,T,D])."""
    import torch
    dt = torch_dtype(wl)
    g = _torch_gen(wl, 4, layer, T, device)
    scale = torch.from_numpy(key_channel_scale(wl, layer)).to(device)[:, None, :]
    k = torch.empty((wl.batch, wl.kv_heads, T, wl.head_dim), dtype=dt, device=device)
    v = torch.empty_like(k)
    for b in range(wl.batch):
        kb = torch.randn((wl.kv_heads, T, wl.head_dim), generator=g, device=device, dtype=torch.float32) * scale
        kb[:, 0, :] *= wl.sink_scale
        k[b] = kb.to(dt)
        v[b] = torch.randn((wl.kv_heads, T, wl.head_dim), generator=g, device=device, dtype=torch.float32).to(dt)
    q = torch.randn((W, wl.batch, wl.q_heads, wl.head_dim), generator=g, device=device, dtype=torch.float32).to(dt)
    return q, k, v
