"""The layer shapes that are tested and benchmarked.

Notation follows the paper (Section 2.2 / 3.1): G groups, S tokens per group,
M model dimension, H hidden dimension of an expert, E experts, C capacity of
one expert within one group.  M=1024 and H=8192 are the paper's Transformer
sizes (Appendix, training details); C = 2S/E is the per-group capacity of
Section 2.2 ("Local group dispatching").
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class MoEConfig:
    name: str
    G: int
    S: int
    M: int
    H: int
    E: int
    C: int
    act_dtype: str = "bf16"        # "f32" or "bf16": x, wi, wo, buffers and y
    seed: int = 20200630
    logit_bias_std: float = 0.0    # > 0: per-expert logit bias (skewed routing)

    @property
    def N(self) -> int:
        return self.G * self.S

    def with_(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = {
    # fp32 throughout; the oracle finishes in well under a second
    "tiny": MoEConfig("tiny", G=1, S=64, M=32, H=64, E=4, C=32, act_dtype="f32",
                      seed=20200631),
    "small": MoEConfig("small", G=4, S=1024, M=512, H=2048, E=16, C=128, seed=20200632),
    # one device's share of a paper-shaped layer
    "paper": MoEConfig("paper", G=8, S=4096, M=1024, H=8192, E=32, C=256, seed=20200633),
    # popular experts overflow: 15-25 % of the top-2 assignments are dropped
    "skewed": MoEConfig("skewed", G=8, S=8192, M=1024, H=4096, E=128, C=128,
                        seed=20200634, logit_bias_std=0.25),
    # many small experts: 17 GB of bf16 expert weights, 16 slots per group
    "many_experts": MoEConfig("many_experts", G=16, S=4096, M=1024, H=8192, E=512, C=16,
                              seed=20200635),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]
