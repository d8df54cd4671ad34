"""The five synthetic workloads (shapes, structure, seeds).

Shapes follow a Qwen2.5-VL-7B-like cache (28 layers, 4 KV heads, head dim 128,
bf16) at the prompt lengths the paper's efficiency section sweeps; contents are
synthetic stand-ins with the structure the paper reports for real caches
(energy concentrated at low token-axis frequencies, a few strongly deviating
KV pairs, layers that differ in their high-frequency share).

Only the hyper-parameters gamma (low-pass cut-off factor) and rho (retention
ratio) are stored here; turning them into integers is the job of whoever
consumes the config (oracle or library), not of the generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple


@dataclass(frozen=True)
class KVConfig:
    name: str
    batch: int
    layers: int
    kv_heads: int
    n_tokens: int
    head_dim: int
    dtype: str                 # "f32" or "bf16" (storage type of K and V)
    gamma: float               # low-pass cut-off factor
    rho: float                 # global retention ratio
    seed: int
    # --- content recipe -----------------------------------------------------
    layout: str = "flat"       # "flat": one smooth signal over all tokens
                               # "blocks": text noise + image blocks
    n_modes: int = 8           # cosine modes per smooth signal
    noise_sigma: float = 0.1   # additive white noise on smooth parts
    text_sigma: float = 1.0    # white-noise text tokens ("blocks" layout)
    n_blocks: int = 0
    block_len: int = 0
    visual_start: int = 0
    drift_delta: float = 0.0   # >0: block bases drift slowly from block to block
    outlier_frac: float = 0.02
    outlier_frac_range: Optional[Tuple[float, float]] = None  # per-layer U(lo,hi)
    outlier_sigma: float = 3.0
    outlier_kind: str = "normal"   # "normal": N(0,sigma^2) vector
                                   # "student": sigma*|t_nu|*N(0,I) vector
    outlier_nu: float = 3.0
    outliers_visual_only: bool = False
    dup_frac: float = 0.0      # fraction of tokens overwritten by a copy of another token

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def units(self) -> int:
        return self.batch * self.layers * self.kv_heads

    @property
    def visual_end(self) -> int:
        return self.visual_start + self.n_blocks * self.block_len

    def scaled(self, **kw) -> "KVConfig":
        """A copy with some fields replaced (used for reduced-size test cases)."""
        from dataclasses import replace
        return replace(self, **kw)


CONFIGS = {
    # 1 layer, single smooth signal + noise + 2 % outliers, fp32, d=64.
    "tiny": KVConfig(
        name="tiny", batch=1, layers=1, kv_heads=2, n_tokens=512, head_dim=64,
        dtype="f32", gamma=0.1, rho=0.2, seed=0,
        layout="flat", outlier_frac=0.02,
    ),
    # 4 layers whose outlier fraction differs, so the budget allocation matters.
    "mid": KVConfig(
        name="mid", batch=1, layers=4, kv_heads=4, n_tokens=4096, head_dim=128,
        dtype="bf16", gamma=0.1, rho=0.2, seed=1,
        layout="flat", outlier_frac_range=(0.005, 0.05),
    ),
    # multi-image prefill: text | 8 image blocks | text
    "qwen_8k": KVConfig(
        name="qwen_8k", batch=1, layers=28, kv_heads=4, n_tokens=8192, head_dim=128,
        dtype="bf16", gamma=0.1, rho=0.2, seed=2,
        layout="blocks", n_blocks=8, block_len=992, visual_start=64,
        outlier_frac=0.03, outliers_visual_only=True,
    ),
    # long multi-image / video context with drifting bases and heavy-tailed outliers
    "long_32k": KVConfig(
        name="long_32k", batch=1, layers=28, kv_heads=4, n_tokens=32768, head_dim=128,
        dtype="bf16", gamma=0.05, rho=0.2, seed=3,
        layout="blocks", n_blocks=32, block_len=1000, visual_start=384,
        drift_delta=0.1, outlier_frac=0.01, outlier_kind="student", outlier_nu=3.0,
    ),
    # batch of 8 independent sequences, duplicated token vectors
    "batch8_16k": KVConfig(
        name="batch8_16k", batch=8, layers=28, kv_heads=4, n_tokens=16384, head_dim=128,
        dtype="bf16", gamma=0.1, rho=0.1, seed=4,
        layout="blocks", n_blocks=8, block_len=2016, visual_start=64,
        outlier_frac=0.03, outliers_visual_only=True, dup_frac=0.005,
    ),
}

ORDER = ["tiny", "mid", "qwen_8k", "long_32k", "batch8_16k"]


def get_config(name: str) -> KVConfig:
    return CONFIGS[name]
