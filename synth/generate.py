"""Seeded generation of one layer's q / k / v token streams.

Recipe (per layer, per sequence), all draws from numpy's counter-based Philox
generator keyed by (seed, layer, seq, kind, token-chunk), so any token range can
be produced without generating the tokens before it:

* per KV head an offset m_h in R^d with entries ~ N(0, 2) (std sqrt 2), shared by
  every token of the head.  It imitates the key anisotropy the paper reports
  (keys nearly collinear with their mean; appendix "Key/query collinearity").
* key   k_t = m_h + z_t, z ~ N(0, 1); each (token, KV head) is an outlier with
  probability `outlier_p`: either the whole key is scaled by `outlier_scale`, or
  (if `outlier_channels` > 0) only that many channels, fixed per head.
* query q_t = N(0, 1) + 0.5 * m_{kv head of the query head}
* value v_t = N(0, 1)
* optional rotary embedding of q and k at the token's prompt position
  (half-split pairing (i, i + d/2), inv_freq_i = theta^(-2i/d), angles in fp64,
  tables cast to fp32), applied after offset/outlier and before rounding.
* round to bf16 (nearest even) and return the bit patterns.

The rotary embedding lives here, in the input recipe, because the eviction
method scores keys as they sit in the cache (Method, "KeyDiff").
"""
from __future__ import annotations

import numpy as np

from .configs import Workload

_CHUNK = 256  # tokens per independently keyed chunk
_KIND_OFFSET, _KIND_K, _KIND_Q, _KIND_V, _KIND_OUTLIER, _KIND_CHANNELS = range(6)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


def _rng(seed: int, layer: int, seq: int, kind: int, chunk: int) -> np.random.Generator:
    key0 = (int(seed) & 0xFFFFFFFF) << 32 | (int(layer) & 0xFFFF) << 16 | (int(seq) & 0xFFFF)
    key1 = (int(kind) & 0xFFFFFFFF) << 32 | (int(chunk) & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=[key0, key1]))


def _normals(seed, layer, seq, kind, t0, t1, inner_shape) -> np.ndarray:
    """Standard normals for tokens [t0, t1), float32, shape (t1 - t0, *inner_shape)."""
    out = np.empty((t1 - t0, *inner_shape), dtype=np.float32)
    c0, c1 = t0 // _CHUNK, (t1 + _CHUNK - 1) // _CHUNK
    for c in range(c0, c1):
        z = _rng(seed, layer, seq, kind, c).standard_normal((_CHUNK, *inner_shape), dtype=np.float32)
        a, b = max(t0, c * _CHUNK), min(t1, (c + 1) * _CHUNK)
        out[a - t0:b - t0] = z[a - c * _CHUNK:b - c * _CHUNK]
    return out


def _uniforms(seed, layer, seq, kind, t0, t1, inner_shape) -> np.ndarray:
    out = np.empty((t1 - t0, *inner_shape), dtype=np.float32)
    c0, c1 = t0 // _CHUNK, (t1 + _CHUNK - 1) // _CHUNK
    for c in range(c0, c1):
        z = _rng(seed, layer, seq, kind, c).random((_CHUNK, *inner_shape), dtype=np.float32)
        a, b = max(t0, c * _CHUNK), min(t1, (c + 1) * _CHUNK)
        out[a - t0:b - t0] = z[a - c * _CHUNK:b - c * _CHUNK]
    return out


def rope_tables(t0: int, T: int, d: int, theta: float):
    """cos and sin of the rotary angles of positions t0 .. t0 + T - 1: float32 [T][d/2]
    (inv_freq_i = theta^(-2i/d), angles in fp64, tables cast to fp32)."""
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = (t0 + np.arange(T, dtype=np.float64))[:, None] * inv_freq[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def apply_rope(x: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotate float32 x[(t, head, d)] by the tables [t][d/2], half-split pairing (i, i + d/2); every
    product and every sum is rounded to float32 on its own (no fused multiply-add)."""
    half = x.shape[-1] // 2
    c, s = cos[:, None, :], sin[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    out = np.empty_like(x)
    out[..., :half] = x1 * c - x2 * s
    out[..., half:] = x2 * c + x1 * s
    return out


def _rope(x: np.ndarray, t0: int, theta: float) -> np.ndarray:
    """Rotate x[(t, head, d)] at positions t0 + t, half-split pairing."""
    cos, sin = rope_tables(t0, x.shape[0], x.shape[-1], theta)
    return apply_rope(x, cos, sin)


def make_layer(w: Workload, seed: int, layer: int = 0, seq: int = 0,
               t0: int = 0, t1: int | None = None, rotate: bool = True):
    """Tokens [t0, t1) of one layer of one sequence.  rotate=False leaves q and k as they are before
    the rotary embedding (for the entry point that applies it itself).

    Returns a dict of bf16 bit patterns (uint16), token-major:
      q [t][n_q_heads][d], k [t][n_kv_heads][d], v [t][n_kv_heads][d]
    plus "offset" (float32 [n_kv_heads][d], the per-head offset m_h).
    """
    if t1 is None:
        t1 = w.prompt_T
    if not (0 <= t0 <= t1):
        raise ValueError("bad token range")
    Hq, Hkv, d, G = w.n_q_heads, w.n_kv_heads, w.head_dim, w.group
    m = _rng(seed, layer, seq, _KIND_OFFSET, 0).standard_normal((Hkv, d), dtype=np.float32)
    m *= np.float32(np.sqrt(2.0))

    k = _normals(seed, layer, seq, _KIND_K, t0, t1, (Hkv, d)) + m[None]
    is_out = _uniforms(seed, layer, seq, _KIND_OUTLIER, t0, t1, (Hkv,)) < np.float32(w.outlier_p)
    if w.outlier_channels > 0:
        crng = _rng(seed, layer, seq, _KIND_CHANNELS, 0)
        for h in range(Hkv):
            ch = crng.choice(d, size=w.outlier_channels, replace=False)
            rows = np.nonzero(is_out[:, h])[0]
            k[np.ix_(rows, [h], ch)] *= np.float32(w.outlier_scale)
    else:
        k[is_out] *= np.float32(w.outlier_scale)

    q = _normals(seed, layer, seq, _KIND_Q, t0, t1, (Hq, d))
    q += np.float32(0.5) * np.repeat(m, G, axis=0)[None]
    v = _normals(seed, layer, seq, _KIND_V, t0, t1, (Hkv, d))

    if w.rope_theta is not None and rotate:
        q = _rope(q, t0, w.rope_theta)
        k = _rope(k, t0, w.rope_theta)

    return {
        "q": f32_to_bf16_bits(q),
        "k": f32_to_bf16_bits(k),
        "v": f32_to_bf16_bits(v),
        "offset": m,
        "t0": t0,
    }


def block_of(arr: np.ndarray, t_start: int, Bt: int) -> np.ndarray:
    """Token-major [t][heads][d] -> one block in the boundary's layout [heads][Bt][d]."""
    return np.ascontiguousarray(arr[t_start:t_start + Bt].transpose(1, 0, 2))
