"""Deterministic synthetic LLM-shaped KV caches.

One NumPy stream per tensor slab: ``default_rng([seed, config_id, b, layer, t])``
with ``t`` = 0 (Q), 1 (K), 2 (V), 3 (auxiliary draws: needle positions, key-norm
factors, sequence lengths).  A slab is one layer of one sequence, so consumers
can stream a large cache layer by layer.

Structure added on top of N(0,1) draws (so that scores look like attention in
a real long-context model rather than white noise):

* sinks: the first ``n_sinks`` tokens of every (layer, KV head) get their key
  shifted along the mean direction of the queries of that KV group by
  ``sink_shift * sqrt(d)`` (4 sigma RMS per coordinate by default);
* needles: ``n_needles`` random positions per (sequence, layer); at each, every
  KV head's key is pushed by ``needle_gain`` along one randomly chosen window
  query of its group;
* optional log-normal key norms (heavy-tailed importance);
* optional per-layer query scale ramp (layer-dependent attention sharpness).

All arithmetic is float32; bf16 workloads are rounded to nearest-even at the
very end and returned as raw uint16 bit patterns, so that every consumer sees
the same bits.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

_T_Q, _T_K, _T_V, _T_AUX = 0, 1, 2, 3
_LEN_LAYER_SLOT = 0xFFFF  # pseudo-layer id for the sequence-length stream


@dataclass(frozen=True)
class WorkloadConfig:
    config_id: int
    name: str
    batch: int
    layers: int
    hq: int
    hkv: int
    head_dim: int
    window: int
    dtype: str                      # "f32" or "bf16"
    keep_percent: int               # retained share of layers*N, in percent
    n: Optional[int] = None         # fixed context length, or None when drawn
    n_range: Optional[Tuple[int, int]] = None   # inclusive range when drawn per sequence
    n_sinks: int = 4
    sink_shift: float = 4.0
    n_needles: int = 64
    needle_gain: float = 8.0
    key_lognormal_sigma: float = 0.0
    q_scale_ramp: Optional[Tuple[float, float]] = None  # (first layer, last layer)
    causal_tail: int = 0            # 1: the window queries are the last M context tokens

    @property
    def group(self) -> int:
        return self.hq // self.hkv


_CONFIGS = {
    0: WorkloadConfig(0, "tiny-f32", 1, 4, 4, 4, 64, 32, "f32", 25, n=1024, n_needles=8),
    1: WorkloadConfig(1, "llama3-8b-32k", 1, 32, 32, 8, 128, 64, "bf16", 20, n=32768),
    2: WorkloadConfig(2, "llama3-8b-128k", 1, 32, 32, 8, 128, 64, "bf16", 10, n=131072),
    3: WorkloadConfig(3, "llama3-8b-varlen-b8", 8, 32, 32, 8, 128, 64, "bf16", 20,
                      n_range=(4096, 32768), key_lognormal_sigma=0.5),
    4: WorkloadConfig(4, "deep-gqa8-64k", 1, 80, 64, 8, 128, 128, "bf16", 15, n=65536,
                      q_scale_ramp=(0.5, 2.0)),
    # the regime of the paper's own evaluation (Section 4.1: 4096-token contexts,
    # Section 4.2: an 8B model of 32 layers, 32/8 heads): many short sequences
    5: WorkloadConfig(5, "llama3-8b-4k-b32", 32, 32, 32, 8, 128, 64, "bf16", 50, n=4096),
    # the other two evaluated models (Section 4.2) at the same 4096-token regime:
    # a 7B model of 28 layers with 28/4 heads (G = 7), a 14B model of 40 layers with
    # 40/8 heads (G = 5); head size 128 in both
    6: WorkloadConfig(6, "qwen2.5-7b-4k-b32", 32, 28, 28, 4, 128, 64, "bf16", 50, n=4096),
    7: WorkloadConfig(7, "qwen3-14b-4k-b32", 32, 40, 40, 8, 128, 64, "bf16", 50, n=4096),
    # task-aware setting (Sections 3.2.1-3.2.2): M is the total number of task tokens of
    # all tasks, here 1024 against a 32k context; and the task-agnostic reading where
    # the window queries are the last M context tokens (causal tail)
    8: WorkloadConfig(8, "llama3-8b-32k-m1024", 1, 32, 32, 8, 128, 1024, "bf16", 20, n=32768),
    9: WorkloadConfig(9, "llama3-8b-32k-causal-tail", 1, 32, 32, 8, 128, 64, "bf16", 20, n=32768,
                      causal_tail=1),
}


def get_config(config_id: int, **overrides) -> WorkloadConfig:
    """Return a named workload; keyword overrides make scaled-down variants."""
    cfg = _CONFIGS[config_id]
    if overrides:
        cfg = replace(cfg, **overrides)
    if cfg.hq % cfg.hkv:
        raise ValueError("hq must be a multiple of hkv")
    return cfg


def seq_lens(cfg: WorkloadConfig, seed: int) -> np.ndarray:
    """Context length of every sequence of the batch (int64 [batch])."""
    if cfg.n is not None:
        return np.full(cfg.batch, cfg.n, dtype=np.int64)
    lo, hi = cfg.n_range
    out = np.empty(cfg.batch, dtype=np.int64)
    for b in range(cfg.batch):
        rng = np.random.default_rng([seed, cfg.config_id, b, _LEN_LAYER_SLOT, _T_AUX])
        out[b] = int(rng.integers(lo, hi, endpoint=True))
    return out


def budget_for(cfg: WorkloadConfig, n: int) -> int:
    """Retained composite tokens for a sequence of length n (integer arithmetic)."""
    return (cfg.keep_percent * cfg.layers * int(n)) // 100


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = (u >> np.uint32(16)) & np.uint32(1)
    bias += np.uint32(0x7FFF)
    bias += u
    bias >>= np.uint32(16)
    return bias.astype(np.uint16)


def make_layer(cfg: WorkloadConfig, seed: int, b: int, layer: int, n: int,
               want_v: bool = True):
    """Draw one (sequence, layer) slab.

    Returns (Q, K, V) with shapes [hq, window, d], [hkv, n, d], [hkv, n, d];
    float32 arrays for "f32" workloads, uint16 bf16 bit patterns for "bf16".
    V is None when ``want_v`` is false.
    """
    d, hq, hkv, g, m = cfg.head_dim, cfg.hq, cfg.hkv, cfg.group, cfg.window
    key = [seed, cfg.config_id, b, layer]
    q = np.random.default_rng(key + [_T_Q]).standard_normal((hq, m, d), dtype=np.float32)
    if cfg.q_scale_ramp is not None:
        lo, hi = cfg.q_scale_ramp
        frac = layer / (cfg.layers - 1) if cfg.layers > 1 else 0.0
        q *= np.float32(lo + (hi - lo) * frac)
    k = np.random.default_rng(key + [_T_K]).standard_normal((hkv, n, d), dtype=np.float32)
    aux = np.random.default_rng(key + [_T_AUX])

    if cfg.key_lognormal_sigma > 0.0:
        z = aux.standard_normal((hkv, n, 1), dtype=np.float32)
        k *= np.exp(np.float32(cfg.key_lognormal_sigma) * z)

    n_sinks = min(cfg.n_sinks, n)
    if n_sinks > 0:
        u = q.reshape(hkv, g * m, d).mean(axis=1)                      # [hkv, d]
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        k[:, :n_sinks, :] += np.float32(cfg.sink_shift * np.sqrt(d)) * u[:, None, :]

    n_needles = min(cfg.n_needles, max(n - n_sinks, 0))
    if n_needles > 0:
        pos = n_sinks + aux.choice(n - n_sinks, size=n_needles, replace=False)
        gi = aux.integers(0, g, size=(n_needles, hkv))
        mi = aux.integers(0, m, size=(n_needles, hkv))
        for j in range(n_needles):
            for h in range(hkv):
                qv = q[h * g + gi[j, h], mi[j, h], :]
                k[h, pos[j], :] += np.float32(cfg.needle_gain) * qv / np.linalg.norm(qv)

    v = None
    if want_v:
        v = np.random.default_rng(key + [_T_V]).standard_normal((hkv, n, d), dtype=np.float32)

    if cfg.dtype == "bf16":
        q = f32_to_bf16_bits(q)
        k = f32_to_bf16_bits(k)
        if v is not None:
            v = f32_to_bf16_bits(v)
    elif cfg.dtype != "f32":
        raise ValueError(f"unknown dtype {cfg.dtype}")
    return q, k, v
