"""Seeded synthetic inputs for the KV-compression pass.

This module only *makes inputs*: it holds none of the method's arithmetic and is
the one piece of code the CPU oracle's tests and the HIP path's tests both use,
so that both sides see identical bits.  numpy only.

The inputs stand in for the prompts the paper runs through real 7-8B models
(Sec. 4.1): the shapes are those models' attention shapes, and the values carry
the two properties the method's ranking relies on (Sec. 3.2 "Initial Ranking"):
a few attention-sink positions at the start and extra weight on recent
positions, plus sparse "heavy" positions in between.

Recipe for one layer (counter-based generator Philox, key = 1000 * config + layer,
one independent stream per tensor and sequence):

  e_h             = random unit vector per (sequence, KV head)
  Q_win[t, hq, :] ~ N(0, 1) + a * sqrt(d) * e_h    t over the last min(w, n) positions; the
                  shared component (a = q_shared) is what makes real window queries agree on
                  where the sinks are; it gives ordinary keys a common logit term ~ N(0, a^2)
  K[p, h, :]      ~ N(0, 1)
  V[p, h, :]      ~ N(0, 1)
  per KV head h:  qbar = mean of the group's window queries, u = qbar / |qbar|,
                  beta(x) = x * sqrt(d) / |qbar|   (a key beta(x) * u gets mean logit x)
  sinks:   K[0..3, h]  = beta(x_sink) * u     x_sink = ln(n)/2 + U(x_sink range), drawn per
                                              (layer, seq, head): the sinks' share of the squared
                                              attention mass then spreads over (0, 1) at any n
  spikes:  K[p, h]    += beta(x_spike) * u    p in a random subset of the non-sink positions
  recency: K[p, h]    += beta(x_rec) * u      p in the last 10 % (config 2 only)

Values are drawn in float32 and rounded once (round-to-nearest-even) to the
config's storage type.  bf16 tensors are carried as uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


# ----------------------------------------------------------------------------
# bf16 <-> fp32 bit conversion (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact upcast of a stored tensor to float64."""
    return bf16_bits_to_f32(x).astype(np.float64) if dtype == "bf16" else x.astype(np.float64)


# ----------------------------------------------------------------------------
# configurations
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    name: str
    layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    dtype: str                      # "fp32" | "bf16"
    batch: int = 1
    context: int = 0                # fixed length (batch of equal sequences) ...
    len_range: tuple = ()           # ... or log-uniform lengths in [lo, hi]
    spike_frac: float = 0.01
    x_spike: float = 2.5
    x_sink: tuple = (1.0, 3.2)      # sink mean logit = ln(n)/2 + U(range), per (layer, seq, head)
    q_shared: float = 1.0           # weight a of the query component shared by a KV head's window
    recency_frac: float = 0.0
    x_rec: float = 0.0
    peaked_first_half: bool = False  # config 3: sequences 0..B/2-1 spiky, the rest flat
    n_sink: int = 4
    threshold: float = 0.01


CONFIGS = {
    0: Config("tiny-fp32", 1, 8, 2, 64, 16, "fp32", context=512, spike_frac=0.02),
    1: Config("llama3-8b-8k", 32, 32, 8, 128, 32, "bf16", context=8192),
    2: Config("qwen2.5-7b-32k", 28, 28, 4, 128, 32, "bf16", context=32768,
              recency_frac=0.10, x_rec=0.5),
    3: Config("mistral-7b-ragged", 32, 32, 8, 128, 32, "bf16", batch=8, len_range=(2048, 32768),
              spike_frac=0.05, x_spike=3.0, peaked_first_half=True),
    4: Config("llama3-8b-128k", 32, 32, 8, 128, 64, "bf16", context=131072, spike_frac=0.005),
    "H": Config("llama3-8b-32k", 32, 32, 8, 128, 32, "bf16", context=32768),
    # the headline shape with the paper's own window, k = 1 (Sec. 4.1 "we set k = 1 in practice")
    "K1": Config("llama3-8b-32k-k1", 32, 32, 8, 128, 1, "bf16", context=32768),
}


@dataclass
class Layer:
    cfg: Config
    q_win: np.ndarray               # [sum_b min(w, n_b), Hq, d]   float32 | uint16(bf16)
    k: np.ndarray                   # [N, Hkv, d]
    v: np.ndarray                   # [N, Hkv, d]
    cu_seqlens: np.ndarray          # int32 [B+1]
    meta: dict = field(default_factory=dict)

    def f64(self, name: str) -> np.ndarray:
        return to_f64(getattr(self, name), self.cfg.dtype)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def seq_lengths(cfg: Config, cfg_id, layer: int = 0) -> np.ndarray:
    """Sequence lengths of the batch (the same for every layer of a config)."""
    if cfg.len_range:
        lo, hi = cfg.len_range
        key = 1000 * (cfg_id if isinstance(cfg_id, int) else 9)
        u = _rng(key, 7).random(cfg.batch)
        return np.round(np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))).astype(np.int64)
    return np.full(cfg.batch, cfg.context, dtype=np.int64)


def make_layer(cfg_id, layer: int = 0, cfg: Config | None = None, lengths=None) -> Layer:
    """Inputs of one transformer layer of configuration `cfg_id`."""
    cfg = cfg or CONFIGS[cfg_id]
    seed = 1000 * (cfg_id if isinstance(cfg_id, int) else 9) + layer
    lens = np.asarray(lengths if lengths is not None else seq_lengths(cfg, cfg_id), dtype=np.int64)
    B = len(lens)
    Hq, Hkv, d, w = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.window
    G = Hq // Hkv
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    N = int(cu[-1])
    wps = np.minimum(w, lens)
    q = np.empty((int(wps.sum()), Hq, d), dtype=np.float32)
    k = np.empty((N, Hkv, d), dtype=np.float32)
    v = np.empty((N, Hkv, d), dtype=np.float32)
    x_sinks = np.zeros((B, Hkv))
    q0 = 0
    for b in range(B):
        n, wp = int(lens[b]), int(wps[b])
        s = int(cu[b])
        qb = _rng(seed, 10 * b + 1).standard_normal((wp, Hq, d), dtype=np.float32)
        if cfg.q_shared:
            e = _rng(seed, 10 * b + 5).standard_normal((Hkv, d))
            e /= np.linalg.norm(e, axis=1, keepdims=True)
            qb += np.repeat(cfg.q_shared * np.sqrt(d) * e, G, axis=0).astype(np.float32)[None]
        kb = _rng(seed, 10 * b + 2).standard_normal((n, Hkv, d), dtype=np.float32)
        v[s:s + n] = _rng(seed, 10 * b + 3).standard_normal((n, Hkv, d), dtype=np.float32)
        aux = _rng(seed, 10 * b + 4)
        peaked = (not cfg.peaked_first_half) or (b < B // 2)
        for h in range(Hkv):
            if n == 0:
                break                                   # an empty sequence has no window and no keys
            qbar = qb[:, h * G:(h + 1) * G, :].astype(np.float64).mean(axis=(0, 1))
            norm = float(np.linalg.norm(qbar))
            u = qbar / norm if norm > 0 else np.zeros(d)
            beta = (lambda x: x * np.sqrt(d) / norm) if norm > 0 else (lambda x: 0.0)
            xs = 0.5 * np.log(max(n, 2)) + aux.uniform(*cfg.x_sink)
            x_sinks[b, h] = xs
            ns = min(cfg.n_sink, n)
            kb[:ns, h, :] = (beta(xs) * u).astype(np.float32)
            n_spk = int(round(cfg.spike_frac * n)) if peaked else 0
            if n_spk > 0 and n > ns:
                pos = ns + aux.choice(n - ns, size=min(n_spk, n - ns), replace=False)
                kb[pos, h, :] += (beta(cfg.x_spike) * u).astype(np.float32)
            if cfg.recency_frac > 0:
                r0 = n - int(round(cfg.recency_frac * n))
                kb[max(r0, ns):, h, :] += (beta(cfg.x_rec) * u).astype(np.float32)
        q[q0:q0 + wp] = qb
        k[s:s + n] = kb
        q0 += wp
    if cfg.dtype == "bf16":
        q, k, v = f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    return Layer(cfg, q, k, v, cu, dict(cfg_id=cfg_id, layer=layer, seed=seed, x_sink=x_sinks,
                                        lengths=lens))


def make_new_queries(cfg_id, layer: int = 0, n_new: int = 64, cfg: Config | None = None, lengths=None) -> np.ndarray:
    """Queries of `n_new` decode positions per sequence, [B, n_new, Hq, d] in the configuration's
    storage type (bf16 as uint16 bit patterns): N(0,1) plus the component the window queries of
    the same layer share, so that the new queries look at the cache the way the window did."""
    cfg = cfg or CONFIGS[cfg_id]
    seed = 1000 * (cfg_id if isinstance(cfg_id, int) else 9) + layer
    lens = np.asarray(lengths if lengths is not None else seq_lengths(cfg, cfg_id), dtype=np.int64)
    B = len(lens)
    Hq, Hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = Hq // Hkv
    q = np.empty((B, n_new, Hq, d), dtype=np.float32)
    for b in range(B):
        qb = _rng(seed, 10 * b + 6).standard_normal((n_new, Hq, d), dtype=np.float32)
        if cfg.q_shared:
            e = _rng(seed, 10 * b + 5).standard_normal((Hkv, d))      # the same draw make_layer uses
            e /= np.linalg.norm(e, axis=1, keepdims=True)
            qb += np.repeat(cfg.q_shared * np.sqrt(d) * e, G, axis=0).astype(np.float32)[None]
        q[b] = qb
    return f32_to_bf16_bits(q) if cfg.dtype == "bf16" else q

