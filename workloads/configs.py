"""The five synthetic MoE-layer shapes (plus one alternative reading of the fifth).

Each stands in for what reaches the expert module of one layer of the models the paper
evaluates (Sec. 5 "Models": Mixtral-8x7B, Mixtral-8x22B, DeepSeek-V2(-Lite)) after
module-based batching has accumulated a large token batch (Sec. 4.2): a [T, H] matrix of
hidden states and a routing distribution.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

BASE_SEED = 250309716


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # accumulated tokens
    H: int            # hidden size
    F: int            # expert FFN width
    E: int            # routed experts
    top_k: int
    num_shared: int   # always-on shared experts (each of width F)
    renormalize: bool  # True: weights renormalised over the selected k (Mixtral); False: raw softmax probs
    bias: str         # "none" | "normal" | "logzipf_rank" | "logzipf_sample"
    seed: int
    routed_scale: float = 1.0

    @property
    def R(self) -> int:
        return self.T * self.top_k

    @property
    def ffn_flops(self) -> int:
        """Algorithmic FLOPs of the grouped SwiGLU FFN: real rows only, no padding."""
        return 6 * (self.T * self.top_k + self.T * self.num_shared) * self.H * self.F

    @property
    def router_flops(self) -> int:
        return 2 * self.T * self.H * self.E


CONFIGS = {
    "C1": MoEConfig("C1", 256, 512, 1024, 8, 2, 0, True, "none", BASE_SEED + 1),
    "C2": MoEConfig("C2", 4096, 4096, 14336, 8, 2, 0, True, "none", BASE_SEED + 2),
    "C3": MoEConfig("C3", 16384, 6144, 16384, 8, 2, 0, True, "normal", BASE_SEED + 3),
    "C4": MoEConfig("C4", 16384, 2048, 1408, 64, 6, 2, False, "none", BASE_SEED + 4),
    "C5": MoEConfig("C5", 32768, 5120, 1536, 160, 6, 2, False, "logzipf_rank", BASE_SEED + 5),
    # Alternative reading of the fifth config's bias: log of *samples* of a Zipf(1.1) law.
    # A handful of experts then take every token and most experts receive none.
    "C5b": MoEConfig("C5b", 32768, 5120, 1536, 160, 6, 2, False, "logzipf_sample", BASE_SEED + 6),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]


def scaled_config(name: str, **overrides) -> MoEConfig:
    """A cut-down copy of a named config (same distributions and seed, other sizes)."""
    return replace(CONFIGS[name], **overrides)
