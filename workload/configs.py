"""Model shapes and workload presets (no arithmetic of the method lives here).

The five benchmark workloads are LLaMA-architecture decoders with fixed-length
random prompts and a fixed number of generated tokens, which is how the paper
builds its own synthetic generation workload (Appendix A, experiment details:
random data at the maximum prompt length, generation stops only at the maximum
length).  The LLaMA-3 rows reproduce the paper's model-configuration table.
"""
from __future__ import annotations

from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    rope_style: int = 1          # 0: pairs (2r, 2r+1); 1: pairs (r, r + head_dim/2)

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers)


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                   # seeds: weights 1000+index, prompts 2000+index
    shape: ModelShape
    batch: int
    prompt_len: int
    gen_len: int
    weights_fp32_master: bool = False   # tiny config draws fp32 weights; others are bf16-valued

    @property
    def max_seq(self) -> int:
        return self.prompt_len + self.gen_len


_TINY = ModelShape(2, 256, 4, 4, 64, 688, 1024)
_L7B = ModelShape(32, 4096, 32, 32, 128, 11008, 32000)
_L13B = ModelShape(40, 5120, 40, 40, 128, 13824, 32000)
_L70B = ModelShape(80, 8192, 64, 8, 128, 28672, 32000)

# The paper's model-configuration table (LLaMA-3 shapes, vocabulary 128256).
LLAMA3_TABLE_SHAPES = {
    "7B": ModelShape(32, 4096, 32, 8, 128, 14336, 128256),
    "13B": ModelShape(40, 5120, 40, 40, 128, 13824, 128256),
    "34B": ModelShape(48, 8192, 64, 8, 128, 22016, 128256),
    "70B": ModelShape(80, 8192, 64, 8, 128, 28672, 128256),
}

PRESETS = {
    "tiny": Workload("tiny", 1, _TINY, 4, 16, 16, weights_fp32_master=True),
    "llama7b": Workload("llama7b", 2, _L7B, 128, 128, 256),
    "llama13b": Workload("llama13b", 3, _L13B, 256, 256, 256),
    "llama7b_long": Workload("llama7b_long", 4, _L7B, 32, 2048, 2048),
    "llama70b": Workload("llama70b", 5, _L70B, 64, 128, 256),
    # the paper's own 7B row (grouped-query attention 32/8, vocabulary 128256) at its base context: prompt 1024,
    # 1024 generated tokens (Appendix A); one GPU's share of the batch
    "llama3_7b": Workload("llama3_7b", 6, LLAMA3_TABLE_SHAPES["7B"], 128, 1024, 1024),
    # the 34B row of the same table at the same context (70.6 GB of weights, 25.8 GB of cache)
    "llama3_34b": Workload("llama3_34b", 7, LLAMA3_TABLE_SHAPES["34B"], 64, 1024, 1024),
}


def preset(name: str) -> Workload:
    return PRESETS[name]
