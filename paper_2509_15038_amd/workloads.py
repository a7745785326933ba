"""Seeded synthetic KV caches and budgets for the five benchmark configurations.

These stand in for the LLaMA-3.1-8B / Mistral-7B caches the paper compresses
(Section 4.1): same shapes (GQA, 8 KV heads x 4 query heads, d = 128), with
channel outliers in K, heavy-tailed token norms in V and a sink-like prefix.
Nothing of the method itself lives here: no sketch, no score, no selection.
Both the CPU oracle's tests and the GPU path's tests draw inputs from this
module so that they see the same bits.

Host generators (numpy, PCG64 seeded by (config, layer, head, tensor)) are the
canonical bits for parity at sizes a CPU can handle.  `device_cache` draws the
same distributions with torch on the GPU for the full-size runs; parity there
copies sampled heads back and feeds those bits to the checker.
"""

from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

__all__ = ["Config", "CONFIGS", "budgets_for", "offsets_for", "host_head",
           "host_cache", "device_cache", "f32_to_bf16_bits", "scaled"]


@dataclass(frozen=True)
class Config:
    name: str
    cfg_id: int
    layers: int
    kv_heads: int
    group: int           # query heads per KV head
    n: int               # tokens
    d: int
    r: int               # sketch dimension
    dtype: str           # "bf16" | "fp32"
    keep: Tuple[float, ...]   # keep fractions; k = floor(keep * n)
    recipe: str          # "c1" (scaled channels + lognormal rows) | "llm"
    prefix_rows: int = 0      # rows 0..prefix_rows-1 scaled by prefix_scale (K and V)
    prefix_scale: float = 1.0
    n_sink: int = 4
    sketch_seed: int = 0xC0DE0001
    dirichlet_total_frac: Optional[float] = None   # C5: per-layer sum of budgets / (H*n)


CONFIGS = {
    "c1": Config("c1", 1, 1, 1, 1, 1024, 128, 32, "fp32", (0.25,), "c1",
                 sketch_seed=0xC0DE0001),
    "c2": Config("c2", 2, 1, 8, 4, 8192, 128, 64, "bf16", (0.20,), "llm",
                 sketch_seed=0xC0DE0002),
    "c3": Config("c3", 3, 32, 8, 4, 32768, 128, 64, "bf16", (0.10, 0.20, 0.50), "llm",
                 sketch_seed=0xC0DE0003),
    "c4": Config("c4", 4, 32, 8, 4, 32768, 128, 64, "bf16", (0.10,), "llm",
                 prefix_rows=64, prefix_scale=10.0, sketch_seed=0xC0DE0004),
    "c5": Config("c5", 5, 32, 8, 4, 131072, 128, 128, "bf16", (0.05,), "llm",
                 sketch_seed=0xC0DE0005, dirichlet_total_frac=0.05),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a configuration with some sizes changed (tests use smaller n/layers)."""
    return replace(cfg, **kw)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def _rng(cfg: Config, layer: int, head: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(
        np.random.SeedSequence([0x5EED, cfg.cfg_id, layer, head, tensor])))


def budgets_for(cfg: Config, keep: Optional[float] = None) -> np.ndarray:
    """int32 [layers*kv_heads] token budgets (sinks included).

    Uniform: k = floor(keep * n).  Dirichlet configs: per layer, shares drawn
    from Dirichlet(1) over the heads, scaled to floor(frac * H * n) tokens,
    rounded by largest remainder, clamped to [0, n] with the sum preserved."""
    L, H, n = cfg.layers, cfg.kv_heads, cfg.n
    if cfg.dirichlet_total_frac is None:
        f = cfg.keep[0] if keep is None else keep
        return np.full(L * H, int(np.floor(f * n + 1e-9)), dtype=np.int32)
    total = int(np.floor(cfg.dirichlet_total_frac * H * n + 1e-9))
    out = np.zeros((L, H), dtype=np.int64)
    for l in range(L):
        rng = _rng(cfg, l, 0, 99)
        share = rng.dirichlet(np.ones(H)) * total
        b = np.floor(share).astype(np.int64)
        rem = total - int(b.sum())
        order = np.argsort(-(share - b), kind="stable")
        b[order[:rem]] += 1
        # clamp to n, hand the excess to the heads with most room
        excess = int(np.sum(np.maximum(b - n, 0)))
        b = np.minimum(b, n)
        while excess > 0:
            room = n - b
            j = int(np.argmax(room))
            take = min(excess, int(room[j]))
            if take == 0:
                break
            b[j] += take
            excess -= take
        out[l] = b
    return out.reshape(-1).astype(np.int32)


def offsets_for(budgets: np.ndarray) -> np.ndarray:
    """int64 [len+1] exclusive prefix sum of the budgets."""
    o = np.zeros(budgets.size + 1, dtype=np.int64)
    o[1:] = np.cumsum(budgets.astype(np.int64))
    return o


def _store(x32: np.ndarray, dtype: str) -> np.ndarray:
    return f32_to_bf16_bits(x32) if dtype == "bf16" else np.ascontiguousarray(x32, np.float32)


def host_head(cfg: Config, layer: int, head: int):
    """(K, V) of one (layer, head) in storage form: uint16 bf16 bits or float32, [n, d]."""
    n, d = cfg.n, cfg.d
    rk, rv = _rng(cfg, layer, head, 0), _rng(cfg, layer, head, 1)
    if cfg.recipe == "c1":
        out = []
        for rng in (rk, rv):
            x = rng.standard_normal((n, d))
            ch = rng.choice(d, size=4, replace=False)
            x[:, ch] *= 8.0
            x *= rng.lognormal(0.0, 0.5, size=(n, 1))
            out.append(x)
        k, v = out
    else:
        c = rk.lognormal(0.0, 1.0, size=(1, d))          # per-channel outlier scales
        k = rk.standard_normal((n, d)) * c
        t = np.abs(rv.standard_t(3.0, size=(n, 1)))       # heavy-tailed row norms
        v = rv.standard_normal((n, d)) * t
    if cfg.prefix_rows:
        p = min(cfg.prefix_rows, n)
        k[:p] *= cfg.prefix_scale
        v[:p] *= cfg.prefix_scale
    return _store(k.astype(np.float32), cfg.dtype), _store(v.astype(np.float32), cfg.dtype)


def host_cache(cfg: Config):
    """(K, V) [layers, kv_heads, n, d] in storage form, generated head by head."""
    L, H = cfg.layers, cfg.kv_heads
    sd = np.uint16 if cfg.dtype == "bf16" else np.float32
    K = np.empty((L, H, cfg.n, cfg.d), dtype=sd)
    V = np.empty((L, H, cfg.n, cfg.d), dtype=sd)
    for l in range(L):
        for h in range(H):
            K[l, h], V[l, h] = host_head(cfg, l, h)
    return K, V


def device_cache(cfg: Config, device="cuda:0"):
    """(K, V) torch tensors [layers, kv_heads, n, d] drawn on the GPU, layer by
    layer, from the same distributions as `host_head` (different bits: torch's
    generator).  Only the "llm" recipe is needed at these sizes."""
    import torch
    assert cfg.recipe == "llm" and cfg.dtype in ("bf16", "fp32")
    L, H, n, d = cfg.layers, cfg.kv_heads, cfg.n, cfg.d
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    K = torch.empty((L, H, n, d), dtype=tdt, device=device)
    V = torch.empty((L, H, n, d), dtype=tdt, device=device)
    g = torch.Generator(device=device)
    g.manual_seed(0x5EED0000 + cfg.cfg_id)
    rows = 8192 if n > 8192 else n
    for l in range(L):
        c = torch.exp(torch.randn((H, 1, d), generator=g, device=device))
        for r0 in range(0, n, rows):
            r1 = min(n, r0 + rows)
            m = r1 - r0
            k = torch.randn((H, m, d), generator=g, device=device) * c
            z = torch.randn((H, m, 3), generator=g, device=device)
            t = torch.randn((H, m, 1), generator=g, device=device)
            t = (t / torch.sqrt((z * z).sum(-1, keepdim=True) / 3.0)).abs()
            v = torch.randn((H, m, d), generator=g, device=device) * t
            if cfg.prefix_rows and r0 < cfg.prefix_rows:
                p = min(cfg.prefix_rows, r1) - r0
                k[:, :p] *= cfg.prefix_scale
                v[:, :p] *= cfg.prefix_scale
            K[l, :, r0:r1] = k.to(tdt)
            V[l, :, r0:r1] = v.to(tdt)
    return K, V
