"""Seeded generators for the five decode workloads and their format conversions.

Random streams are counter-based (numpy's Philox) and keyed by
(1000 * config id + stream id, sequence index), so every consumer that asks for
the same (config, stream, sequence) sees the same numbers no matter the order of
calls.  Stream ids: 0 keys, 1 values, 2 queries, 3 channel scales, 4 appended
keys, 5 appended values, 6 planted positions, 7 query drift noise, 8 block means of the
supplementary cache with positional locality.

Values are drawn in fp32 and, for bf16 workloads, rounded to the nearest bf16
(ties to even) so the fp32 arrays handed to the CPU side and the 16-bit patterns
uploaded to the GPU hold exactly the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
from numpy.random import Generator, Philox

STREAM_K, STREAM_V, STREAM_Q, STREAM_SCALE = 0, 1, 2, 3
STREAM_APPEND_K, STREAM_APPEND_V, STREAM_PLANT, STREAM_DRIFT = 4, 5, 6, 7
STREAM_LOCAL = 8

# The five workloads.  "dist": "iid" = N(0,1) entries; "channel" = N(0,1) entries
# times a per-channel scale exp(0.5 g), g ~ N(0,1), with four seeded channels
# multiplied by 10 (heavy-tailed key norms, a few dominant channels).
CONFIGS = {
    1: dict(name="single_head_n4096_f32", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=128,
            n=4096, dtype="f32", dist="iid", qualify_frac=0.02, planted=8, steps=1),
    2: dict(name="gqa32x8_n32768_bf16", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128,
            n=32768, dtype="bf16", dist="channel", qualify_frac=0.01, steps=1),
    3: dict(name="gqa32x8_n131072_bf16_drift256", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128,
            n=131072, dtype="bf16", dist="channel", qualify_frac=0.005, steps=256),
    4: dict(name="gqa32x8_n32768_b16_bf16", batch=16, n_q_heads=32, n_kv_heads=8, head_dim=128,
            n=32768, dtype="bf16", dist="channel", qualify_frac=0.02, steps=1),
    5: dict(name="gqa32x8_prompt16384_append4096_bf16", batch=1, n_q_heads=32, n_kv_heads=8,
            head_dim=128, n=16384, dtype="bf16", dist="channel", tau_below_max=8.0, steps=4096),
}


def _rng(config_id: int, stream: int, seq: int = 0) -> Generator:
    return Generator(Philox(key=[1000 * int(config_id) + int(stream), int(seq)]))


# --------------------------------------------------------------------------- formats
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array whose every value is the nearest bf16-representable number."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


def _bits_of_exact(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of an fp32 array whose values are already bf16-representable: the upper
    halves of the words (checked: the lower halves must be zero)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.bitwise_and(u, np.uint32(0xFFFF)).any():      # not exact after all: round
        return f32_to_bf16_bits(x).reshape(x.shape)
    return (u >> np.uint32(16)).astype(np.uint16).reshape(x.shape)


# --------------------------------------------------------------------------- caches
@dataclass
class KVCache:
    """K, V as fp32 arrays [batch][n_kv_heads][n][head_dim] holding values exact in `dtype`."""
    K: np.ndarray
    V: np.ndarray
    dtype: str
    channel_scale: np.ndarray | None = None     # [batch][n_kv_heads][head_dim] or None
    meta: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.K.shape[2]

    def K_bits(self) -> np.ndarray:
        assert self.dtype == "bf16"
        return _bits_of_exact(self.K)

    def V_bits(self) -> np.ndarray:
        assert self.dtype == "bf16"
        return _bits_of_exact(self.V)


def _channel_scales(config_id: int, seq: int, n_kv_heads: int, d: int) -> np.ndarray:
    g = _rng(config_id, STREAM_SCALE, seq)
    s = np.exp(0.5 * g.standard_normal((n_kv_heads, d), dtype=np.float32)).astype(np.float32)
    for h in range(n_kv_heads):
        hot = g.choice(d, size=4, replace=False)
        s[h, hot] *= np.float32(10.0)
    return s


def _draw_rows(config_id, stream, seq, shape, dist, scales, dtype):
    x = _rng(config_id, stream, seq).standard_normal(shape, dtype=np.float32)
    if dist == "channel" and scales is not None:
        x *= scales[:, None, :]
    elif dist not in ("iid", "channel"):
        raise ValueError(dist)
    if dtype == "bf16":
        x = round_to_bf16(x)
    return x


def make_cache(config_id: int, *, n: int | None = None, batch: int | None = None,
               n_kv_heads: int | None = None) -> KVCache:
    """The prompt-time KV cache of a workload.  n / batch / n_kv_heads override the
    workload's size (for reduced test cases); the distribution and seeds stay the same."""
    c = CONFIGS[config_id]
    n = c["n"] if n is None else int(n)
    batch = c["batch"] if batch is None else int(batch)
    hkv = c["n_kv_heads"] if n_kv_heads is None else int(n_kv_heads)
    d = c["head_dim"]
    K = np.empty((batch, hkv, n, d), dtype=np.float32)
    V = np.empty((batch, hkv, n, d), dtype=np.float32)
    scales = np.empty((batch, hkv, d), dtype=np.float32) if c["dist"] == "channel" else None
    def one(b):
        sc = None
        if scales is not None:
            sc = _channel_scales(config_id, b, hkv, d)
            scales[b] = sc
        K[b] = _draw_rows(config_id, STREAM_K, b, (hkv, n, d), c["dist"], sc, c["dtype"])
        V[b] = _draw_rows(config_id, STREAM_V, b, (hkv, n, d), "iid", None, c["dtype"])
    # every sequence has streams of its own, so the sequences can be drawn side by side
    if batch > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(batch, 8)) as pool:
            list(pool.map(one, range(batch)))
    else:
        one(0)
    return KVCache(K=K, V=V, dtype=c["dtype"], channel_scale=scales,
                   meta=dict(config=config_id, name=c["name"]))


def make_local_cache(config_id: int, *, block: int = 64, spread: float = 3.0, noise: float = 0.05,
                     n: int | None = None, batch: int | None = None,
                     n_kv_heads: int | None = None) -> KVCache:
    """Supplementary workload (not one of the five): keys with positional locality.  Every run of
    `block` consecutive tokens shares a mean drawn from N(0, spread^2) per coordinate and adds
    N(0, noise^2) of its own, so neighbouring keys are close in key space and groups of consecutive
    keys have tight bounding balls.  Values as in the base workload.  Same shapes as config_id."""
    c = CONFIGS[config_id]
    n = c["n"] if n is None else int(n)
    batch = c["batch"] if batch is None else int(batch)
    hkv = c["n_kv_heads"] if n_kv_heads is None else int(n_kv_heads)
    d = c["head_dim"]
    nb = (n + block - 1) // block
    K = np.empty((batch, hkv, n, d), dtype=np.float32)
    V = np.empty((batch, hkv, n, d), dtype=np.float32)
    for b in range(batch):
        g = _rng(config_id, STREAM_LOCAL, b)
        means = g.standard_normal((hkv, nb, d), dtype=np.float32) * np.float32(spread)
        K[b] = np.repeat(means, block, axis=1)[:, :n]
        K[b] += np.float32(noise) * g.standard_normal((hkv, n, d), dtype=np.float32)
        V[b] = _draw_rows(config_id, STREAM_V, b, (hkv, n, d), "iid", None, c["dtype"])
    if c["dtype"] == "bf16":
        K = round_to_bf16(K)
    return KVCache(K=K, V=V, dtype=c["dtype"], channel_scale=None,
                   meta=dict(config=config_id, name=c["name"] + "_local_keys"))


def make_append_stream(config_id: int, steps: int, cache: KVCache) -> tuple[np.ndarray, np.ndarray]:
    """Keys/values produced during decoding: [steps][batch][n_kv_heads][head_dim], same
    distribution as the prompt cache (same channel scales)."""
    c = CONFIGS[config_id]
    batch, hkv, _, d = cache.K.shape
    k_new = np.empty((steps, batch, hkv, d), dtype=np.float32)
    v_new = np.empty((steps, batch, hkv, d), dtype=np.float32)
    for b in range(batch):
        sc = cache.channel_scale[b] if cache.channel_scale is not None else None
        k = _draw_rows(config_id, STREAM_APPEND_K, b, (hkv, steps, d), c["dist"], sc, c["dtype"])
        v = _draw_rows(config_id, STREAM_APPEND_V, b, (hkv, steps, d), "iid", None, c["dtype"])
        k_new[:, b] = k.transpose(1, 0, 2)
        v_new[:, b] = v.transpose(1, 0, 2)
    return k_new, v_new


# --------------------------------------------------------------------------- queries
def make_queries(config_id: int, *, batch: int | None = None, n_q_heads: int | None = None,
                 step: int = 0, exact_bf16: bool | None = None) -> np.ndarray:
    """q ~ N(0,1): fp32 [batch][n_q_heads][head_dim].  For bf16 workloads the values are
    rounded to bf16-representable numbers so a bf16 and an fp32 reading of q agree."""
    c = CONFIGS[config_id]
    batch = c["batch"] if batch is None else int(batch)
    hq = c["n_q_heads"] if n_q_heads is None else int(n_q_heads)
    q = np.empty((batch, hq, c["head_dim"]), dtype=np.float32)
    for b in range(batch):
        g = Generator(Philox(key=[1000 * config_id + STREAM_Q, (b << 32) | step]))
        q[b] = g.standard_normal((hq, c["head_dim"]), dtype=np.float32)
    if exact_bf16 is None:
        exact_bf16 = c["dtype"] == "bf16"
    return round_to_bf16(q) if exact_bf16 else q


def drift_queries(config_id: int, steps: int, *, rho: float = 0.9, noise: float = 0.44,
                  batch: int | None = None, n_q_heads: int | None = None) -> np.ndarray:
    """Autoregressive query path q_t = rho q_{t-1} + noise N(0,1) (stationary for
    rho^2 + noise^2 ~ 1): fp32 [steps][batch][n_q_heads][head_dim], bf16-representable."""
    c = CONFIGS[config_id]
    q0 = make_queries(config_id, batch=batch, n_q_heads=n_q_heads, exact_bf16=False)
    out = np.empty((steps,) + q0.shape, dtype=np.float32)
    g = _rng(config_id, STREAM_DRIFT, 0)
    cur = q0
    for t in range(steps):
        if t > 0:
            cur = (np.float32(rho) * cur
                   + np.float32(noise) * g.standard_normal(q0.shape, dtype=np.float32))
        out[t] = cur
    return round_to_bf16(out) if c["dtype"] == "bf16" else out


# --------------------------------------------------------------------------- thresholds
def tau_for_count(scores: np.ndarray, k: int) -> np.ndarray:
    """Threshold midway between the k-th and (k+1)-th largest entries along the last axis,
    so exactly k entries are >= it (when those two order statistics differ).
    k = 0 gives a value above the maximum; k >= n gives -inf."""
    s = np.asarray(scores)
    n = s.shape[-1]
    if k >= n:
        return np.full(s.shape[:-1], -np.inf, dtype=np.float32)
    if k <= 0:
        return (s.max(axis=-1) + np.abs(s.max(axis=-1)) * 1e-3 + 1.0).astype(np.float32)
    part = np.partition(s, (n - k - 1, n - k), axis=-1)
    hi = part[..., n - k].astype(np.float64)
    lo = part[..., n - k - 1].astype(np.float64)
    return (0.5 * (hi + lo)).astype(np.float32)


def tau_for_fraction(scores: np.ndarray, frac: float) -> np.ndarray:
    n = np.asarray(scores).shape[-1]
    return tau_for_count(scores, int(np.ceil(frac * n)))


def plant_rows(K: np.ndarray, rows: np.ndarray, factors: np.ndarray, dtype: str) -> None:
    """Rescale the given rows of one head's key matrix [n][d] in place (row i by factors[i]),
    re-rounding to the storage format.  The caller derives the factors from scores it owns."""
    K[rows] = K[rows] * np.asarray(factors, dtype=np.float32)[:, None]
    if dtype == "bf16":
        K[rows] = round_to_bf16(K[rows])


def planted_positions(config_id: int, n: int, count: int) -> np.ndarray:
    return np.sort(_rng(config_id, STREAM_PLANT, 0).choice(n, size=count, replace=False))
