"""Seeded synthetic inputs for one DASH attention layer.

This module holds no arithmetic of the method: it only draws random tensors of
the shapes and value distributions of the benchmark workloads and rounds them
to the storage type. Both the GPU path and the CPU oracle's tests take their
inputs from here, so both see bit-identical values.

Workloads (stand-ins for long prompts on a Qwen2.5-7B / Llama-3-8B shaped layer;
only shapes and the heavy-tailed score structure are imitated):
  hidden rows  x_t = g_t * exp(mu + sigma z_t), g_t ~ N(0, I), z_t ~ N(0, 1)
  q, k, v      ~ N(0, 1)
  W_o          ~ N(0, 1/hidden)       (second argument is the variance)
  active_idx   sorted seeded uniform subset of 0..N-1 of size n
The per-row lognormal factor makes the relative score ||U_t|| / ||x_t|| strongly
skewed: most rows small, a sparse long tail, as in Fig. 1 / Fig. 8 of the paper.

Values are returned as float32 numpy arrays that are exactly representable in
the storage type (bf16 or fp32), so `astype(float64)` and a cast to bf16 both
reproduce them without rounding.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    dtype: str            # "bf16" or "f32": storage type of x, q, k, v, w_o
    N: int                # original prompt length
    n: int                # active tokens entering the layer
    d: int                # hidden size
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    halt_frac: float      # fraction of active rows halted by the percentile threshold
    seed: int
    causal: bool = True
    # row-norm mixture: list of (weight, mu, sigma) of the lognormal row factor
    row_scale: tuple = ((1.0, 0.0, 1.5),)

    @property
    def D_a(self) -> int:
        return self.n_q_heads * self.head_dim


# The five benchmark configurations.
CONFIGS = {
    "tiny_f32": LayerConfig("tiny_f32", "f32", 512, 512, 256, 4, 1, 64, 0.50, seed=0),
    "qwen_8k": LayerConfig("qwen_8k", "bf16", 8192, 8192, 3584, 28, 4, 128, 0.60, seed=1),
    "qwen_32k_half": LayerConfig("qwen_32k_half", "bf16", 32768, 16384, 3584, 28, 4, 128, 0.30, seed=2),
    "qwen_32k_chain": LayerConfig("qwen_32k_chain", "bf16", 32768, 32768, 3584, 28, 4, 128, 0.20, seed=3),
    "llama_128k_40": LayerConfig("llama_128k_40", "bf16", 131072, 52428, 4096, 32, 8, 128, 0.50, seed=4,
                                 row_scale=((0.8, 1.0, 0.5), (0.2, 0.0, 1.5))),
}


def scaled(cfg: LayerConfig, n: int, N: int | None = None, **kw) -> LayerConfig:
    """Same layer shape at another length (for parity cases the oracle finishes in seconds)."""
    if N is None:
        N = max(n, int(round(n * cfg.N / cfg.n)))
    return replace(cfg, name=f"{cfg.name}@n{n}", n=n, N=N, **kw)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    r &= np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _store(a: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(dtype)


def make_active_idx(N: int, n: int, seed: int) -> np.ndarray:
    if n == N:
        return np.arange(N, dtype=np.int32)
    perm = _rng(seed, 5).permutation(N)[:n]
    return np.sort(perm).astype(np.int32)


def make_hidden(cfg: LayerConfig, n: int | None = None) -> np.ndarray:
    n = cfg.n if n is None else n
    g = _rng(cfg.seed, 0).standard_normal((n, cfg.d), dtype=np.float32)
    z = _rng(cfg.seed, 6).standard_normal(n)
    if len(cfg.row_scale) == 1:
        _, mu, sigma = cfg.row_scale[0]
        f = np.exp(mu + sigma * z)
    else:
        u = _rng(cfg.seed, 7).random(n)
        edges = np.cumsum([w for w, _, _ in cfg.row_scale])
        comp = np.searchsorted(edges, u, side="right").clip(0, len(cfg.row_scale) - 1)
        mus = np.array([m for _, m, _ in cfg.row_scale])[comp]
        sig = np.array([s for _, _, s in cfg.row_scale])[comp]
        f = np.exp(mus + sig * z)
    g *= f.astype(np.float32)[:, None]
    return _store(g, cfg.dtype)


def make_layer_inputs(cfg: LayerConfig) -> dict:
    """x [n,d], q [n,Hq,dh], k,v [n,Hkv,dh], w_o [Hq*dh, d], active_idx [n] int32."""
    n = cfg.n
    x = make_hidden(cfg)
    q = _store(_rng(cfg.seed, 1).standard_normal((n, cfg.n_q_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
    k = _store(_rng(cfg.seed, 2).standard_normal((n, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
    v = _store(_rng(cfg.seed, 3).standard_normal((n, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32), cfg.dtype)
    w_o = _rng(cfg.seed, 4).standard_normal((cfg.D_a, cfg.d), dtype=np.float32)
    w_o *= np.float32(1.0 / np.sqrt(cfg.d))
    w_o = _store(w_o, cfg.dtype)
    return dict(x=x, q=q, k=k, v=v, w_o=w_o, active_idx=make_active_idx(cfg.N, n, cfg.seed))


def make_projection_weights(cfg: LayerConfig, layer: int) -> dict:
    """Per-layer W_q [d, Hq*dh], W_k, W_v [d, Hkv*dh], W_o [Hq*dh, d] ~ N(0, 1/d) for the layer chain."""
    out = {}
    shapes = dict(w_q=(cfg.d, cfg.D_a), w_k=(cfg.d, cfg.n_kv_heads * cfg.head_dim),
                  w_v=(cfg.d, cfg.n_kv_heads * cfg.head_dim), w_o=(cfg.D_a, cfg.d))
    for s, (name, shp) in enumerate(shapes.items()):
        w = _rng(cfg.seed, 100 + 10 * layer + s).standard_normal(shp, dtype=np.float32)
        w *= np.float32(1.0 / np.sqrt(cfg.d))
        out[name] = _store(w, cfg.dtype)
    return out


def make_ffn_weights(cfg: LayerConfig, layer: int, m: int) -> dict:
    """Per-layer gated feed-forward weights: W_gate, W_up [d, m] ~ N(0, 1/d), W_down [m, d] ~ N(0, 1/m)."""
    out = {}
    for s, (name, shp, fan) in enumerate((("w_gate", (cfg.d, m), cfg.d), ("w_up", (cfg.d, m), cfg.d),
                                          ("w_down", (m, cfg.d), m))):
        w = _rng(cfg.seed, 500 + 10 * layer + s).standard_normal(shp, dtype=np.float32)
        w *= np.float32(1.0 / np.sqrt(fan))
        out[name] = _store(w, cfg.dtype)
    return out


def sample_rows(n: int, count: int, seed: int, tile: int = 128) -> np.ndarray:
    """Query rows for a row-sampled check: both ends, rows around the first tile
    boundaries, the last ragged tile, the rest seeded-uniform. Sorted, unique."""
    fixed = list(range(min(8, n))) + list(range(max(0, n - 8), n))
    for b in (1, 2, 3):
        for off in (-1, 0, 1):
            r = b * tile + off
            if 0 <= r < n:
                fixed.append(r)
    last_tile = (n - 1) // tile * tile
    fixed += [r for r in (last_tile - 1, last_tile, last_tile + 1) if 0 <= r < n]
    fixed = np.unique(np.array(fixed, dtype=np.int64))
    if count > fixed.size and n > fixed.size:
        rest = np.setdiff1d(np.arange(n, dtype=np.int64), fixed)
        extra = _rng(seed, 9).choice(rest, size=min(rest.size, count - fixed.size), replace=False)
        fixed = np.concatenate([fixed, extra])
    return np.sort(fixed).astype(np.int64)


def percentile_tau(scores: np.ndarray, halt_frac: float):
    """Threshold that halts the h = floor(halt_frac * n) lowest scores: the fp32
    midpoint between the h-th and (h+1)-th smallest. Returns (tau as float, h).
    The matching TopK call keeps n - h rows."""
    s = np.sort(np.asarray(scores, dtype=np.float64))
    n = s.shape[0]
    h = int(np.floor(halt_frac * n))
    if h <= 0:
        return 0.0, 0
    if h >= n:
        return float(np.float32(np.inf)), n
    tau = np.float32(0.5 * (s[h - 1] + s[h]))
    if not (s[h - 1] < float(tau)):
        tau = np.nextafter(np.float32(s[h - 1]), np.float32(np.inf))
        if not (s[h - 1] < float(tau)):
            tau = np.nextafter(tau, np.float32(np.inf))
    return float(tau), h
