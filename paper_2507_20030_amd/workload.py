"""Seeded synthetic workloads: Llama-shaped K/V caches, kept-bin masks, decode inputs.

Holds shapes, distributions and index sets only -- none of the method's
arithmetic -- so that the CPU oracle tests and the GPU path can draw the very
same inputs.  Values are generated with torch's seeded generators on the
requested device and rounded to the storage dtype before anyone consumes them.
"""
from __future__ import annotations

import dataclasses
from typing import List

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    n_layers: int
    batch: int
    n_kv_heads: int
    group: int            # query heads per KV head
    head_dim: int
    L: int                # transformed prefill tokens = DFT length M (prefill holds n_sink + L + n_recent)
    n_bins: int           # kept bins per layer
    steps: int            # decode steps (append + attention)
    dtype: str            # "f32" or "bf16"
    mask: str             # "low" or "mixed" (half the layers low band, half low + mid groups)
    outlier_channels: int = 0
    n_sink: int = 0       # first tokens kept exact (attention sinks)
    n_recent: int = 0     # newest tokens kept exact (recent window)
    outlier_scale: float = 20.0
    seed: int = 0

    @property
    def n_q_heads(self) -> int:
        return self.n_kv_heads * self.group

    @property
    def n_prefill(self) -> int:
        return self.n_sink + self.L + self.n_recent

    @property
    def n_slices(self) -> int:
        return self.n_layers * self.batch * self.n_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


CONFIGS = {
    # configs[0..4] of the baseline description
    "cfg1": Config("cfg1", 1, 1, 8, 1, 128, 1024, 64, 16, "f32", "low"),
    "cfg2": Config("cfg2", 32, 1, 8, 4, 128, 8192, 2048, 256, "bf16", "low"),
    "cfg3": Config("cfg3", 32, 8, 8, 4, 128, 32768, 4096, 512, "bf16", "mixed"),
    "cfg4": Config("cfg4", 32, 1, 8, 4, 128, 131072, 4096, 1024, "bf16", "low"),
    "cfg5": Config("cfg5", 80, 16, 8, 8, 128, 16384, 1638, 128, "bf16", "mixed", outlier_channels=4),
    # cfg2 with the paper's exact windows (Sec. 5.1: 10 sink tokens, 50 recent tokens)
    "cfg2w": Config("cfg2w", 32, 1, 8, 4, 128, 8192, 2048, 256, "bf16", "low", n_sink=10, n_recent=50),
    # the same windows cut OUT of an 8192-token context: M = 8192 - 60 = 8132 is not a power of two (25 % of the bins)
    "cfg2x": Config("cfg2x", 32, 1, 8, 4, 128, 8132, 2033, 256, "bf16", "low", n_sink=10, n_recent=50),
    # cfg3's shape keeping 25 % of the bins (the paper's largest ratio, Sec. 5.1): 8192 per layer, beyond the 4096 the
    # register-resident FFT kernels take
    "cfg3b": Config("cfg3b", 32, 8, 8, 4, 128, 32768, 8192, 512, "bf16", "mixed"),
    # cfg3's shape with the paper's windows cut out of a 32768-token context: M = 32708 = 4 x 8177
    "cfg3x": Config("cfg3x", 32, 8, 8, 4, 128, 32708, 4088, 512, "bf16", "mixed", n_sink=10, n_recent=50),
}


def _seed(cfg: Config, *parts: int) -> int:
    h = np.uint64(0x9E3779B97F4A7C15) ^ np.uint64(cfg.seed + 1)
    with np.errstate(over="ignore"):
        for p in parts:
            h = (h ^ np.uint64(p + 0x632BE5AB)) * np.uint64(0xBF58476D1CE4E5B9)
            h ^= h >> np.uint64(29)
    return int(h & np.uint64(0x7FFFFFFFFFFFFFFF))


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


# ----------------------------------------------------------------------------- masks
def mask_low(n: int) -> np.ndarray:
    return np.arange(n, dtype=np.int32)


def mask_low_mid(M: int, n: int, rng: np.random.Generator, group: int = 64) -> np.ndarray:
    """Low band plus `group`-wide blocks scattered over the mid band [n_low, M/2)."""
    n_mid = n // (2 * group)
    n_low = n - group * n_mid
    first = -(-n_low // group)                       # first group-aligned start at or above n_low
    starts = np.arange(first, (M // 2) // group) * group
    n_mid = min(n_mid, len(starts))
    n_low = n - group * n_mid
    pick = rng.choice(starts, size=n_mid, replace=False) if n_mid else np.zeros(0, np.int64)
    bins = np.concatenate([np.arange(n_low), *(np.arange(s, s + group) for s in np.sort(pick))])
    bins = np.unique(bins).astype(np.int32)
    assert len(bins) == n and bins.max() < M
    return bins


def layer_bins(cfg: Config) -> List[np.ndarray]:
    """Sorted kept bins of every layer (host int32 arrays)."""
    if cfg.mask == "low":
        return [mask_low(cfg.n_bins) for _ in range(cfg.n_layers)]
    rng = np.random.default_rng(_seed(cfg, 17))
    order = rng.permutation(cfg.n_layers)
    kinds = np.empty(cfg.n_layers, dtype=bool)         # True = low + mid
    kinds[order[: cfg.n_layers // 2]] = False
    kinds[order[cfg.n_layers // 2:]] = True
    return [mask_low_mid(cfg.L, cfg.n_bins, rng) if kinds[l] else mask_low(cfg.n_bins)
            for l in range(cfg.n_layers)]


# ---------------------------------------------------------------------------- values
_SCALE_CACHE: dict = {}


def k_channel_scale(cfg: Config, layer: int, device) -> torch.Tensor:
    """Per (kv head, channel) scale of K: log-uniform in [0.1, 10], optional x20 outliers."""
    key = (cfg, layer, str(device))
    if key not in _SCALE_CACHE:
        _SCALE_CACHE[key] = _k_channel_scale(cfg, layer, device)
    return _SCALE_CACHE[key]


def _k_channel_scale(cfg: Config, layer: int, device) -> torch.Tensor:
    g = _gen("cpu", _seed(cfg, 3, layer))
    s = 10.0 ** (2.0 * torch.rand((cfg.n_kv_heads, cfg.head_dim), generator=g) - 1.0)
    for h in range(cfg.n_kv_heads):
        if cfg.outlier_channels:
            idx = torch.randperm(cfg.head_dim, generator=g)[: cfg.outlier_channels]
            s[h, idx] *= cfg.outlier_scale
    return s.to(device)


def prefill_layer(cfg: Config, layer: int, device):
    """K, V of one layer, [batch, n_kv_heads, n_sink + L + n_recent, head_dim] in the storage dtype."""
    g = _gen(device, _seed(cfg, 5, layer))
    shape = (cfg.batch, cfg.n_kv_heads, cfg.n_prefill, cfg.head_dim)
    K = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    K *= k_channel_scale(cfg, layer, device)[None, :, None, :]
    K = K.to(cfg.torch_dtype)
    V = torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(cfg.torch_dtype)
    return K, V


def prefill_tensors(cfg: Config, device):
    """K, V of all layers, [n_layers, batch, n_kv_heads, n_sink + L + n_recent, head_dim]."""
    shape = (cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.n_prefill, cfg.head_dim)
    K = torch.empty(shape, device=device, dtype=cfg.torch_dtype)
    V = torch.empty(shape, device=device, dtype=cfg.torch_dtype)
    for l in range(cfg.n_layers):
        K[l], V[l] = prefill_layer(cfg, l, device)
    return K, V


def decode_step(cfg: Config, step: int, device):
    """Token K/V [n_layers, batch, n_kv_heads, d] and queries [n_layers, batch, n_q_heads, d]."""
    g = _gen(device, _seed(cfg, 7, step))
    kv_shape = (cfg.n_layers, cfg.batch, cfg.n_kv_heads, cfg.head_dim)
    key = (cfg, "all", str(device))
    if key not in _SCALE_CACHE:
        _SCALE_CACHE[key] = torch.stack([k_channel_scale(cfg, l, device) for l in range(cfg.n_layers)])[:, None]
    scale = _SCALE_CACHE[key]
    tk = (torch.randn(kv_shape, generator=g, device=device, dtype=torch.float32) * scale).to(cfg.torch_dtype)
    tv = torch.randn(kv_shape, generator=g, device=device, dtype=torch.float32).to(cfg.torch_dtype)
    q = torch.randn((cfg.n_layers, cfg.batch, cfg.n_q_heads, cfg.head_dim), generator=g, device=device,
                    dtype=torch.float32).to(cfg.torch_dtype)
    return tk, tv, q


def sample_slices(cfg: Config, n: int = 8):
    """(layer, batch, kv_head) triples used for parity and for timing the oracle:
    first, last, and seeded picks covering both mask kinds."""
    total = cfg.n_slices
    if total <= n:
        idx = list(range(total))
    else:
        rng = np.random.default_rng(_seed(cfg, 23))
        idx = sorted({0, total - 1, *rng.choice(total, size=n - 2, replace=False).tolist()})
    spl = cfg.batch * cfg.n_kv_heads
    return [(i // spl, (i % spl) // cfg.n_kv_heads, i % cfg.n_kv_heads) for i in idx]
