"""Named workload shapes.

The shapes follow the model families the paper evaluates (Llama-3.1-8B,
Llama-3.2-3B, Qwen-2.5-7B; Experiments, "Experimental Setup"), its block size
B = 128 (and 64 / 256 in the block-size ablation) and its 2K-8K cache budgets.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional


@dataclass(frozen=True)
class Workload:
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prompt_T: int          # prompt length in tokens
    block_B: int           # prompt block size
    budget_N: int          # cache budget
    batch: int = 1         # independent sequences
    n_layers: int = 1      # layers the bench sums over
    rope_theta: Optional[float] = None   # None: no rotation
    outlier_p: float = 0.02              # probability a (token, kv head) key is an outlier
    outlier_scale: float = 4.0           # factor applied to an outlier key
    outlier_channels: int = 0            # 0: whole key scaled; >0: that many fixed channels per head
    decode_steps: int = 0                # >0: decode workload (B = 1 after a full cache)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def small(self, **kw) -> "Workload":
        """A reduced copy (same distribution) for tests."""
        return replace(self, **kw)


CONFIGS = {
    # correctness config: the oracle runs the whole prompt in seconds
    "toy": Workload("toy", 4, 1, 64, 1024, 32, 256),
    "llama32_3b": Workload("llama32_3b", 24, 8, 128, 16384, 128, 4096, n_layers=28, rope_theta=500000.0),
    # headline: timed per block step, summed over 32 layers with a fresh seed per layer
    "llama31_8b": Workload("llama31_8b", 32, 8, 128, 32768, 128, 8192, n_layers=32,
                           rope_theta=500000.0),
    "qwen25_7b": Workload("qwen25_7b", 28, 4, 128, 32768, 256, 8192, n_layers=28, rope_theta=1.0e6,
                          outlier_p=0.01, outlier_scale=8.0, outlier_channels=4),
    "decode_8b": Workload("decode_8b", 32, 8, 128, 8192 + 1024, 1, 8192, batch=16,
                          rope_theta=500000.0, decode_steps=1024),
}


def get_config(name: str) -> Workload:
    try:
        return CONFIGS[name]
    except KeyError:
        raise KeyError(f"unknown workload {name!r}; have {sorted(CONFIGS)}") from None
