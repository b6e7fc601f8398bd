"""The synthetic workload shapes.

Shapes follow the evaluated models' expert geometry (paper Table 2: Mixtral-8x7B
with 8 experts / top-2 / 336 MiB per bf16 expert; DeepSeek-V2-Lite-like with 64
experts / top-6 / 16.5 MiB per expert) and the batch range of the evaluation
(Section 5.1: batch 4-64, short decode).  Values are synthetic: the paper's
datasets and trained weights are not reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class MoEConfig:
    name: str
    T: int            # tokens in the batch
    H: int            # hidden size
    E: int            # routed experts
    k: int            # experts activated per token
    F: int            # expert FFN width
    S: int            # always-on shared experts
    dtype: str        # "f32" or "bf16" (storage of X, Wr, expert weights)
    bias: str         # "none" | "normal" | "zipf"
    bias_scale: float = 0.0
    w_std: float = 0.02
    seed: int = 0
    layers: int = 1
    steps: int = 1

    @property
    def A(self) -> int:
        """Routed (token, slot) assignments."""
        return self.T * self.k

    @property
    def rows(self) -> int:
        """Rows the grouped FFN produces: routed assignments + shared rows."""
        return self.T * self.k + self.S * self.T

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def expert_bytes(self) -> int:
        """Three matrices per expert (Section 4.4), no biases."""
        return 3 * self.H * self.F * self.itemsize

    def with_(self, **kw) -> "MoEConfig":
        return replace(self, **kw)


CONFIGS = {
    # configs[0]: tiny fp32 layer, router bias N(0,1)
    "c1_tiny": MoEConfig("c1_tiny", T=8, H=256, E=8, k=2, F=512, S=0,
                         dtype="f32", bias="normal", bias_scale=1.0),
    # configs[1]: Mixtral-8x7B-shaped decode layer, router bias N(0,0.5)
    "c2_mixtral": MoEConfig("c2_mixtral", T=64, H=4096, E=8, k=2, F=14336, S=0,
                            dtype="bf16", bias="normal", bias_scale=0.5),
    # configs[2]: fine-grained experts + 4 shared, Zipf(1.1) popularity prior
    "c3_finegrained": MoEConfig("c3_finegrained", T=128, H=2048, E=60, k=4,
                                F=1408, S=4, dtype="bf16", bias="zipf",
                                bias_scale=1.1),
    # configs[3]: DeepSeek-V2-Lite-shaped prefill, 4 x 512 tokens, no bias
    "c4_dsv2lite_prefill": MoEConfig("c4_dsv2lite_prefill", T=2048, H=2048,
                                     E=64, k=6, F=1408, S=2, dtype="bf16",
                                     bias="none"),
    # configs[4]: 32-layer Mixtral-shaped stack, batch 32, 16 decode steps
    "c5_stack": MoEConfig("c5_stack", T=32, H=4096, E=8, k=2, F=14336, S=0,
                          dtype="bf16", bias="normal", bias_scale=0.5,
                          layers=32, steps=16),
    # widening case: Qwen3-30B-A3B-shaped decode layer (Table 2: 128 experts,
    # top-8, 9 MiB per bf16 expert = 3 x 2048 x 768 x 2 bytes), batch 64
    "c6_qwen3_a3b": MoEConfig("c6_qwen3_a3b", T=64, H=2048, E=128, k=8, F=768,
                              S=0, dtype="bf16", bias="normal", bias_scale=0.5),
}


def get_config(name: str, **overrides) -> MoEConfig:
    cfg = CONFIGS[name]
    return cfg.with_(**overrides) if overrides else cfg
