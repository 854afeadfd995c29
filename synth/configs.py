"""The synthetic MoE-layer workloads (shapes of the paper's Table 1 models and of two further
public MoE shapes).  Only shapes and distribution switches live here.  Configs 1-5 are the
benchmark's workload list; config 6 is the third model of the paper's Table 1 (the fine-grained
shape its fused kernel is motivated by, section 3.4.3), added as a further parity workload."""
from dataclasses import dataclass, field
from typing import Tuple


@dataclass(frozen=True)
class LayerConfig:
    index: int                 # 1..6, also the leading term of every seed
    name: str
    hidden: int                # H
    n_experts: int             # E routed experts
    inter: int                 # I, SwiGLU intermediate size
    top_k: int                 # k
    group_size: int            # g, int4 group length along the input dimension
    n_shared: int = 0          # S always-on shared experts (bf16 in both passes)
    renormalize: int = 1       # routing weights renormalised over the selected k
    verify_tokens: Tuple[int, ...] = (4,)   # K+1 values exercised
    router: str = "plain"      # plain | zipf | ar1   (how logits get their structure)
    n_layers: int = 1          # depth of the stack the workload runs
    n_resident: int = 0        # experts per layer resident in the slot table (0 = all)
    bench_layers: int = 1      # distinct layers the benchmark rotates over

    @property
    def params_per_expert(self) -> int:
        return 3 * self.hidden * self.inter

    @property
    def bf16_expert_bytes(self) -> int:
        return 2 * self.params_per_expert

    @property
    def int4_expert_bytes(self) -> int:
        p = self.params_per_expert
        return p // 2 + (p // self.group_size) * 4


CONFIGS = (
    LayerConfig(1, "tiny", 256, 8, 512, 2, 32, verify_tokens=(4,), bench_layers=4),
    LayerConfig(2, "phi", 4096, 16, 6400, 2, 128, verify_tokens=(5,), router="zipf",
                bench_layers=32),
    LayerConfig(3, "mixtral", 4096, 8, 14336, 2, 128, verify_tokens=(2, 4, 8), bench_layers=8),
    LayerConfig(4, "qwen3", 2048, 128, 768, 8, 64, verify_tokens=(8,), router="ar1",
                bench_layers=8),
    LayerConfig(5, "dsv2lite", 2048, 64, 1408, 6, 128, n_shared=2, verify_tokens=(6,),
                n_layers=27, n_resident=16, bench_layers=27),
    # Qwen1.5-MoE-A2.7B shape: 60 experts, top-4, one shared expert of 4x the width = 4 of width I
    LayerConfig(6, "qwen15", 2048, 60, 1408, 4, 128, n_shared=4, verify_tokens=(6,), router="ar1",
                n_layers=24, bench_layers=8),
)


def config_by_name(name: str) -> LayerConfig:
    for c in CONFIGS:
        if c.name == name or str(c.index) == str(name):
            return c
    raise KeyError(name)
