"""The five synthetic layer configurations (shapes and input recipes only).

Notation follows the paper: T tokens, d model dim, ffn hidden dim, E experts,
top-k, N logical ranks, c replica slots per rank, S = N*c slots, P = T*k pairs.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int
    d: int
    ffn: int
    E: int
    k: int
    N: int
    c: int
    dtype: str            # "f32" | "bf16"
    act: str              # "gelu" | "swiglu"
    seed: int
    steps: int = 1
    ranking_seed: Optional[int] = None  # seed of the expert popularity ranking if not `seed`
    bias: str = "zipf"    # "normal": b ~ N(0, bias_param); "zipf": b = -s ln(rank+1)
    bias_param: float = 1.0
    reshuffle_every: int = 0          # redraw the popularity ranking every n steps (0 = never)
    s_range: Optional[Tuple[float, float]] = None   # per-step Zipf exponent drawn uniformly
    replica_counts: Optional[Tuple[int, ...]] = None  # fixed allocation (else Eq. 1 on step-0 loads)
    placement: str = "mro"            # "mro" | "spread"
    f: int = 1                        # fault-tolerance threshold used for the allocation
    # post-failure scenario: start from the plan of `base` and drop these ranks
    base: Optional[str] = None
    base_N: int = 0
    base_c: int = 0
    drop_ranks: Tuple[int, ...] = field(default_factory=tuple)

    @property
    def S(self) -> int:
        return self.N * self.c

    @property
    def P(self) -> int:
        return self.T * self.k


CONFIGS = {
    "c1_tiny": LayerConfig(
        name="c1_tiny", T=256, d=128, ffn=256, E=8, k=2, N=4, c=4,
        dtype="f32", act="gelu", seed=0, bias="normal", bias_param=0.5,
        replica_counts=(3, 3, 2, 2, 2, 2, 1, 1), placement="spread"),
    "c2_mixtral": LayerConfig(
        name="c2_mixtral", T=8192, d=4096, ffn=14336, E=8, k=2, N=8, c=2,
        dtype="bf16", act="swiglu", seed=2, bias="zipf", bias_param=1.0),
    "c3_gptmoe": LayerConfig(
        name="c3_gptmoe", T=16384, d=2048, ffn=8192, E=32, k=2, N=8, c=6,
        dtype="bf16", act="gelu", seed=3, steps=20, bias="zipf", bias_param=1.2,
        reshuffle_every=5),
    "c4_finegrained": LayerConfig(
        name="c4_finegrained", T=16384, d=2048, ffn=1408, E=64, k=6, N=16, c=8,
        dtype="bf16", act="swiglu", seed=4, bias="zipf", bias_param=1.1),
    "c5_postfailure": LayerConfig(
        name="c5_postfailure", T=16384, d=2048, ffn=8192, E=32, k=2, N=6, c=8,
        dtype="bf16", act="gelu", seed=5, steps=100, bias="zipf", bias_param=1.2,
        s_range=(0.8, 1.5), base="c3_gptmoe", base_N=8, base_c=6, drop_ranks=(6, 7),
        # the traffic keeps the popularity ranking the re-plan was proportioned for: the base
        # config's ranking at step 0 (its seed, epoch 0); only the Zipf exponent changes per step
        ranking_seed=3),
}

ORDER = ["c1_tiny", "c2_mixtral", "c3_gptmoe", "c4_finegrained", "c5_postfailure"]


def get_config(name: str) -> LayerConfig:
    return CONFIGS[name]


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of `cfg` with some fields replaced (used for reduced-size parity cases)."""
    from dataclasses import replace
    return replace(cfg, **kw)
