"""Counter-based seeded generators for keys, values and step-correlated queries.

Recipe
  * K, V: i.i.d. N(0,1); four fixed outlier channels multiplied by 8; then
    rounded (nearest-even) to the storage type.
  * q:   q_0 ~ N(0,1); q_t = rho * q_{t-1} + q_noise * N(0,1) in fp32, the fp32
    state carried on unrounded, each emitted q_t rounded to the storage type.
    With shift_every > 0, every such step q_t is a fresh N(0,1) draw.
  * every stream is keyed by (seed, layer, request, kind) through Philox, so a
    single layer or request can be regenerated alone.

Everything is returned as float32 arrays whose values are exactly representable
in the storage type, next to the uint16 bit patterns handed to the GPU.
"""
from __future__ import annotations

import numpy as np

OUTLIER_CHANNELS = (7, 43, 71, 101)
OUTLIER_SCALE = 8.0

_KIND_KV_PREFIX = 1
_KIND_KV_DECODE = 2
_KIND_QUERY = 3


def _rng(seed: int, layer: int, request: int, kind: int) -> np.random.Generator:
    key = np.array([np.uint64(seed), np.uint64((layer << 40) | (request << 8) | kind)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 -> uint16 bit patterns of fp16 / bf16, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
        return ((u + r) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def decode(bits: np.ndarray, dtype: str) -> np.ndarray:
    """uint16 bit patterns of fp16 / bf16 -> float32 (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "fp16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(dtype)


def _kv_draw(rng: np.random.Generator, n_tokens: int, n_kv: int, d: int, dtype: str):
    out = []
    for _ in range(2):
        x = rng.standard_normal((n_tokens, n_kv, d), dtype=np.float32)
        x[..., list(OUTLIER_CHANNELS)] *= np.float32(OUTLIER_SCALE)
        bits = encode(x, dtype)
        out.append((decode(bits, dtype), bits))
    return out


def kv_prefix(wl, layer: int, request: int, n_tokens: int | None = None):
    """Cached context of one (layer, request): ((K, Kbits), (V, Vbits)), each [n_tokens, n_kv, d]."""
    n = wl.ctx if n_tokens is None else n_tokens
    return _kv_draw(_rng(wl.seed, layer, request, _KIND_KV_PREFIX), n, wl.n_kv_heads, wl.head_dim, wl.dtype)


def kv_decode_tokens(wl, layer: int, request: int, n_steps: int | None = None):
    """The token appended at each decode step: ((K, Kbits), (V, Vbits)), each [n_steps, n_kv, d]."""
    n = wl.steps if n_steps is None else n_steps
    return _kv_draw(_rng(wl.seed, layer, request, _KIND_KV_DECODE), n, wl.n_kv_heads, wl.head_dim, wl.dtype)


def query_stream(wl, layer: int, request: int, n_steps: int | None = None):
    """Step-correlated queries: (q, qbits), each [n_steps, n_q, d]."""
    n = wl.steps if n_steps is None else n_steps
    rng = _rng(wl.seed, layer, request, _KIND_QUERY)
    noise = rng.standard_normal((n, wl.n_q_heads, wl.head_dim), dtype=np.float32)
    rho = np.float32(wl.rho)
    c = np.float32(wl.q_noise)
    state = noise[0].copy()
    q = np.empty_like(noise)
    q[0] = state
    for t in range(1, n):
        if wl.shift_every and t % wl.shift_every == 0:
            state = noise[t].copy()
        else:
            state = rho * state + c * noise[t]
        q[t] = state
    bits = encode(q, wl.dtype)
    return decode(bits, wl.dtype), bits
