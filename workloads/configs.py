"""Workload shapes: one entry per benchmark configuration.

The shapes follow the models the paper evaluates (Llama-3-8B, Qwen3-8B, a
70B-class target; Sec. 6.1 "Tasks and Datasets") and its default
hyper-parameters N=60, mu=0.03, K=10 (Sec. 6.1 "Implementation Details").
The value structure of the logits follows the paper's own synthetic recipe
(App. E.6: Zipfian next-token distributions) and the two entropy regimes of
Sec. 5.2.1 "Intuition" (peaked rows vs flat rows).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    B: int            # independent sequences
    V: int            # draft vocabulary width
    logits_dtype: str  # "f32" or "bf16" (storage type of a logits row)
    K: int            # per-row candidate cap and width of the top-K init layer
    N: int            # node budget, root included
    Dmax: int         # cap on the number of layers
    mu: float         # confidence-gate threshold
    Hq: int
    Hkv: int
    Dh: int
    L: int            # prefix KV length per sequence
    # logits recipe: ("gauss", lo, hi) -> beta~U[lo,hi] per row times N(0,1);
    # a tuple of per-sequence recipes means sequence b uses recipe[b % len].
    # ("zipf_mix", alpha, sigma): even node ids Zipf-peaked, odd near-uniform.
    recipe: Tuple = field(default=("gauss", 0.5, 4.0))
    seed: int = 20260107

    @property
    def N_pad(self) -> int:
        return (self.N + 63) // 64 * 64

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elem_bytes(self) -> int:
        return 4 if self.logits_dtype == "f32" else 2


CONFIGS = {
    # tiny step the CPU oracle finishes in well under a second
    "c1": WorkloadConfig("c1-tiny", B=1, V=1024, logits_dtype="f32", K=2, N=16, Dmax=6,
                         mu=0.03, Hq=4, Hkv=4, Dh=64, L=128,
                         recipe=("gauss", 0.5, 4.0)),
    # Llama-3-8B-shaped: the configuration the headline metric is quoted on
    "c2": WorkloadConfig("c2-llama3-8b", B=1, V=128256, logits_dtype="bf16", K=10, N=60,
                         Dmax=12, mu=0.03, Hq=32, Hkv=8, Dh=128, L=2048,
                         recipe=("gauss", 0.5, 8.0)),
    # Qwen3-8B-shaped, four sequences: two low-temperature, two high-temperature
    "c3": WorkloadConfig("c3-qwen3-8b-x4", B=4, V=151936, logits_dtype="bf16", K=8, N=128,
                         Dmax=16, mu=0.03, Hq=32, Hkv=8, Dh=128, L=4096,
                         recipe=(("gauss", 6.0, 8.0), ("gauss", 6.0, 8.0),
                                 ("gauss", 0.5, 1.0), ("gauss", 0.5, 1.0))),
    # 70B-shaped verification on one GPU (all 64 heads, no tensor-parallel split)
    "c4": WorkloadConfig("c4-70b", B=1, V=128256, logits_dtype="bf16", K=10, N=60,
                         Dmax=12, mu=0.03, Hq=64, Hkv=8, Dh=128, L=8192,
                         recipe=("gauss", 0.5, 8.0)),
    # stress: sixteen sequences, Zipf-peaked / near-uniform rows, long prefix
    "c5": WorkloadConfig("c5-stress", B=16, V=151936, logits_dtype="bf16", K=16, N=256,
                         Dmax=24, mu=0.03, Hq=32, Hkv=8, Dh=128, L=16384,
                         recipe=("zipf_mix", 1.2, 0.05)),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name.lower()]
