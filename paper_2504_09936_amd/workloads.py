"""Seeded synthetic inputs for the KeepKV hot path.

This module only draws random tensors of the shapes and statistics of the five
workload configurations (head layouts, context length, budget ratio taken from
the paper's setup: Sec. 1 for the 70B / batch-128 / 8K example, Sec. 4.1 for
the model families and the 10 % / 20 % ratios).  It contains none of the
method's arithmetic; it is the one module both the CPU oracle's tests and the
HIP path's tests read, so that both see bit-identical inputs.

All draws come from numpy's counter-based Philox generator keyed by
(seed, tensor tag, step), so any tensor can be regenerated independently.
Values are rounded once (round-to-nearest-even) to the storage dtype and
returned as float32 arrays holding exactly representable values; `to_bf16_bits`
gives the uint16 payload that is uploaded to the device.
"""
from __future__ import annotations

import math
import zlib
from dataclasses import dataclass, replace

import numpy as np

__all__ = [
    "Workload", "CONFIGS", "budget_of", "round_bf16", "to_bf16_bits", "from_bf16_bits",
    "round_storage", "make_cache", "make_query", "make_token", "rng_for",
]


# --------------------------------------------------------------------------- dtype plumbing
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 payload (uint16), round-to-nearest-even, NaN kept quiet."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = np.isnan(x)
    out = rounded.astype(np.uint16)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bfloat16 payload (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float values to the nearest bfloat16, returned as float32."""
    return from_bf16_bits(to_bf16_bits(np.asarray(x, dtype=np.float32)))


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an array to the storage dtype ('f32' or 'bf16'); result is float32."""
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# --------------------------------------------------------------------------- configurations
def budget_of(context: int, ratio: float) -> int:
    """Slots kept per (batch, kv-head): ceil(ratio * context) (52 of 512, 820 of 8192)."""
    return int(math.ceil(ratio * context - 1e-9))


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # storage of Q, K, V, O: 'f32' or 'bf16'
    context: int          # N: tokens in the cache before the first compression
    ratio: float          # budget / context
    period: int           # P: decode steps between compression events
    steps: int            # decode steps after the first compression
    window: int           # observation passes over the uncompressed cache (w + 1)
    key_model: str        # 'outlier', 'mixture', 'decay', 'ar1'
    n_outlier: int = 0
    outlier_scale: float = 1.0
    query_model: str = "direction"   # 'mean' (Tiny) or 'direction'
    alpha: float = 0.9               # EMA decay (the paper gives no value)
    threshold: float = 0.8           # merging threshold T (Sec. 4.1)
    n_sink: int = 4                  # always-kept first tokens (App. B.3)

    @property
    def budget(self) -> int:
        return budget_of(self.context, self.ratio)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_recent(self) -> int:
        """Recent window : heavy hitters = 4 : 1 within the non-sink budget (App. B.3)."""
        return (4 * (self.budget - self.n_sink)) // 5

    @property
    def capacity(self) -> int:
        return max(self.context, self.budget + self.period)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    def scaled(self, **kw) -> "Workload":
        """A smaller instance of the same recipe (parity tests)."""
        return replace(self, **kw)


CONFIGS = {
    "tiny": Workload("tiny", 1, 4, 4, 64, "f32", 512, 0.10, 32, 64, 32,
                     "outlier", n_outlier=2, outlier_scale=8.0, query_model="mean"),
    "llama3_8b": Workload("llama3_8b", 8, 32, 8, 128, "bf16", 8192, 0.10, 64, 256, 32,
                          "outlier", n_outlier=4, outlier_scale=6.0),
    "llama3_8b_20": Workload("llama3_8b_20", 8, 32, 8, 128, "bf16", 8192, 0.20, 64, 256, 32,
                             "outlier", n_outlier=4, outlier_scale=6.0),
    "long_32k": Workload("long_32k", 1, 32, 8, 128, "bf16", 32768, 0.10, 128, 512, 32, "mixture"),
    "llama3_70b": Workload("llama3_70b", 128, 64, 8, 128, "bf16", 8192, 0.10, 64, 64, 8, "decay"),
    "stress": Workload("stress", 16, 32, 8, 128, "bf16", 16384, 0.05, 16, 1024, 32, "ar1"),
}


# --------------------------------------------------------------------------- random streams
def rng_for(seed: int, tag: str, *index: int) -> np.random.Generator:
    """Independent Philox stream for (seed, tensor tag, integer indices)."""
    key = np.array([int(seed) & 0xFFFFFFFFFFFFFFFF, zlib.crc32(tag.encode())], dtype=np.uint64)
    ctr = np.zeros(4, dtype=np.uint64)
    for i, v in enumerate(index[:3]):
        ctr[i + 1] = int(v) & 0xFFFFFFFFFFFFFFFF   # negative steps (observation window) wrap
    return np.random.Generator(np.random.Philox(key=key, counter=ctr))


_AR_RHO = 0.98
_N_CLUSTER = 64


def _outlier_channels(w: Workload, seed: int) -> np.ndarray:
    """[B, Hkv, n_outlier] channel ids, drawn once per (batch, kv head)."""
    g = rng_for(seed, "outlier_channels")
    out = np.empty((w.batch, w.n_kv_heads, max(w.n_outlier, 1)), dtype=np.int64)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            out[b, h] = g.choice(w.head_dim, size=max(w.n_outlier, 1), replace=False)
    return out


def _channel_scale(w: Workload) -> np.ndarray:
    """1/f-style per-channel standard deviation, mean variance 1 ('decay' keys)."""
    s = 1.0 / (1.0 + np.arange(w.head_dim, dtype=np.float64))
    return s / math.sqrt(float(np.mean(s * s)))


def _cluster_centres(w: Workload, seed: int):
    g = rng_for(seed, "cluster_centres")
    mu = g.standard_normal((w.batch, w.n_kv_heads, _N_CLUSTER, w.head_dim))
    mu /= np.linalg.norm(mu, axis=-1, keepdims=True)
    nu = g.standard_normal((w.batch, w.n_kv_heads, _N_CLUSTER, w.head_dim))
    return mu, nu


def _query_centres(w: Workload, seed: int) -> np.ndarray:
    """[B, Hq, D]: the fixed direction each query head looks along."""
    g = rng_for(seed, "query_centres")
    u = g.standard_normal((w.batch, w.n_q_heads, w.head_dim))
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    return u


def _keys_values(w: Workload, seed: int, tag: str, n: int, first_pos: int,
                 prev=None) -> tuple[np.ndarray, np.ndarray]:
    """Draw n consecutive (k, v) rows per (batch, kv head), float64, before rounding."""
    B, H, D = w.batch, w.n_kv_heads, w.head_dim
    g = rng_for(seed, tag, first_pos)
    k = g.standard_normal((B, H, n, D))
    v = g.standard_normal((B, H, n, D))
    if w.key_model == "outlier":
        ch = _outlier_channels(w, seed)
        for b in range(B):
            for h in range(H):
                k[b, h][:, ch[b, h][: w.n_outlier]] *= w.outlier_scale
    elif w.key_model == "decay":
        k *= _channel_scale(w)
    elif w.key_model == "mixture":
        mu, nu = _cluster_centres(w, seed)
        which = g.integers(0, _N_CLUSTER, size=(B, H, n))
        bi = np.arange(B)[:, None, None]
        hi = np.arange(H)[None, :, None]
        # noise of total norm ~0.3 around a unit centre, then scaled to norm ~sqrt(D)
        k = (mu[bi, hi, which] + k * (0.3 / math.sqrt(D))) * math.sqrt(D)
        v = v + nu[bi, hi, which]
    elif w.key_model == "ar1":
        c = math.sqrt(1.0 - _AR_RHO ** 2)
        pk = np.zeros((B, H, D)) if prev is None else prev[0]
        pv = np.zeros((B, H, D)) if prev is None else prev[1]
        for i in range(n):
            if prev is None and i == 0:
                pass  # stationary start: k_0 ~ N(0, I)
            else:
                k[:, :, i] = _AR_RHO * pk + c * k[:, :, i]
                v[:, :, i] = _AR_RHO * pv + c * v[:, :, i]
            pk, pv = k[:, :, i], v[:, :, i]
    else:
        raise ValueError(w.key_model)
    return k, v


def make_cache(w: Workload, seed: int = 0):
    """Prefill cache of w.context tokens: K, V as float32 [B, Hkv, N, D], storage-rounded."""
    k, v = _keys_values(w, seed, "prefill", w.context, 0)
    if w.query_model == "mean":
        # token 0 is an attention sink: its key points along the mean query of its head
        mu = _query_centres(w, seed)[:, :: w.group] * math.sqrt(w.head_dim)
        k[:, :, 0] = 3.0 * mu / np.linalg.norm(mu, axis=-1, keepdims=True)
    return round_storage(k, w.dtype), round_storage(v, w.dtype)


def make_query(w: Workload, seed: int, step: int) -> np.ndarray:
    """Query of decode (or observation-window) step `step`: float32 [B, Hq, D]."""
    u = _query_centres(w, seed)
    g = rng_for(seed, "query", step)
    xi = g.standard_normal(u.shape)
    D = w.head_dim
    if w.query_model == "mean":
        q = u * math.sqrt(D) + 0.25 * xi
    else:
        q = 3.0 * math.sqrt(D) * (u + 0.25 * xi / math.sqrt(D))
    return round_storage(q, w.dtype)


def make_token(w: Workload, seed: int, step: int, prev=None):
    """(k_t, v_t) appended at decode step `step`: float32 [B, Hkv, D] each.

    For the AR(1) key model `prev` = (k, v) of the previous token, unrounded or rounded.
    """
    k, v = _keys_values(w, seed, "decode", 1, step + 1,
                        prev=None if prev is None else (np.asarray(prev[0], np.float64),
                                                        np.asarray(prev[1], np.float64)))
    return round_storage(k[:, :, 0], w.dtype), round_storage(v[:, :, 0], w.dtype)
