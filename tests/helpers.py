"""Shared plumbing for the GPU parity tests: upload bf16 bit patterns, run the
oracle and the HIP path side by side on the same seeded blocks."""
from __future__ import annotations

import numpy as np

from synth import bf16_bits_to_f32, block_of


def to_dev(bits: np.ndarray, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def to_bits(t) -> np.ndarray:
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bf16_out_to_f32(t) -> np.ndarray:
    return bf16_bits_to_f32(to_bits(t))


def blocks(data, B, T=None):
    """Yield (t, Bt, q, k, v) with q/k/v in the boundary's [1][heads][Bt][d] layout (bits)."""
    T = data["k"].shape[0] if T is None else T
    for t in range(0, T, B):
        Bt = min(B, T - t)
        yield t, Bt, block_of(data["q"], t, Bt)[None], block_of(data["k"], t, Bt)[None], block_of(data["v"], t, Bt)[None]


def rows_by_position(cache):
    """(positions, K bits, V bits) of the HIP cache, every head sorted by position."""
    ln = cache.len
    pos = cache.positions().cpu().numpy()
    K = to_bits(cache.key_rows()[:, :, :ln])
    V = to_bits(cache.value_rows()[:, :, :ln])
    order = np.argsort(pos, axis=-1, kind="stable")
    pos_s = np.take_along_axis(pos, order, axis=-1)
    K_s = np.take_along_axis(K, order[..., None], axis=2)
    V_s = np.take_along_axis(V, order[..., None], axis=2)
    return pos_s, K_s, V_s


SCORE_RTOL, SCORE_ATOL = 1e-5, 1e-7      # scores: 1e-5 relative (+ a floor for scores near zero)
ATTN_ATOL = 2e-2                          # attention, bf16 I/O against the fp64 oracle
