"""Model shapes and workload recipes.

The paper benchmarks trained 4-bit checkpoints of the Qwen3 and Llama-3.2
families (evaluation setup, Table 1) and a 1 -> 16 concurrent-request sweep
(continuous-batching scaling paragraph, Fig. 2).  Those checkpoints and prompts
are not available, so each workload takes the public *shape* of one of those
models and replaces values with seeded distributions.
"""
from dataclasses import dataclass, field, asdict
from typing import Optional, Tuple


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e4
    qk_norm: bool = False
    n_experts: int = 0        # 0 = dense SwiGLU MLP
    top_k: int = 0
    expert_ffn: int = 0
    tie_lm_head: bool = False

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def dense_weight_bytes(self) -> int:
        """bf16 bytes of every matrix streamed once per decode step."""
        H, d = self.hidden, self.head_dim
        attn = H * self.q_dim + 2 * H * self.kv_dim + self.q_dim * H
        if self.n_experts:
            mlp = self.n_experts * H  # router only; experts are data dependent
        else:
            mlp = 3 * H * self.ffn
        return 2 * (self.n_layers * (attn + mlp) + self.vocab * H)

    def expert_bytes(self) -> int:
        return 2 * 3 * self.hidden * self.expert_ffn if self.n_experts else 0

    def kv_bytes_per_token(self) -> int:
        return self.n_layers * 2 * self.kv_dim * 2

    def as_dict(self):
        return asdict(self)


CONFIGS = {
    "tiny": ModelConfig("tiny", 2, 256, 4, 2, 64, 688, 1024,
                        rms_eps=1e-6, rope_theta=1e4),
    "qwen3_0p6b": ModelConfig("qwen3_0p6b", 28, 1024, 16, 8, 128, 3072, 151936,
                              rope_theta=1e6, qk_norm=True, tie_lm_head=True),
    "llama32_3b": ModelConfig("llama32_3b", 28, 3072, 24, 8, 128, 8192, 128256,
                              rope_theta=5e5, tie_lm_head=True),
    "qwen3_8b": ModelConfig("qwen3_8b", 36, 4096, 32, 8, 128, 12288, 151936,
                            rope_theta=1e6, qk_norm=True),
    "qwen3_30b_a3b": ModelConfig("qwen3_30b_a3b", 48, 2048, 32, 4, 128, 0, 151936,
                                 rope_theta=1e6, qk_norm=True,
                                 n_experts=128, top_k=8, expert_ffn=768),
    # The 8B shape cut to 4 layers: every kernel at its real size, a tenth of the weights.
    "qwen3_8b_l4": ModelConfig("qwen3_8b_l4", 4, 4096, 32, 8, 128, 12288, 151936,
                               rope_theta=1e6, qk_norm=True),
    # The 30B-A3B shape cut to 4 layers: every kernel runs at its real size while
    # weights stay at 5 GB (the 48-layer model is 61 GB).
    "qwen3_30b_a3b_l4": ModelConfig("qwen3_30b_a3b_l4", 4, 2048, 32, 4, 128, 0, 151936,
                                    rope_theta=1e6, qk_norm=True,
                                    n_experts=128, top_k=8, expert_ffn=768),
    # Not a benchmark shape: the tiny model with every contraction length a multiple of 128,
    # which the 4-bit weight format needs.
    "tiny_q4": ModelConfig("tiny_q4", 2, 256, 4, 2, 64, 768, 1000,
                           rms_eps=1e-6, rope_theta=1e4, qk_norm=True),
    # Not a benchmark shape: a few-layer MoE small enough for the oracle.
    "tiny_moe": ModelConfig("tiny_moe", 2, 256, 4, 2, 64, 0, 1024,
                            qk_norm=True, n_experts=8, top_k=2, expert_ffn=96),
}


@dataclass(frozen=True)
class Workload:
    """One decode workload: a model shape plus the batch structure."""
    name: str
    model: str
    batch: int
    block_size: int
    steps: int
    # explicit contexts, or a (lo, hi) uniform draw
    contexts: Optional[Tuple[int, ...]] = None
    context_range: Optional[Tuple[int, int]] = None
    shared_prefix: int = 0        # tokens; multiple of block_size
    n_sharers: int = 0
    seed_weights: int = 0
    seed_kv: int = 1
    seed_tokens: int = 2
    seed_blocks: int = 3

    @property
    def cfg(self) -> ModelConfig:
        return CONFIGS[self.model]


WORKLOADS = {
    "cfg0": Workload("cfg0", "tiny", 2, 16, 8, contexts=(32, 17)),
    "cfg1": Workload("cfg1", "qwen3_0p6b", 1, 16, 128, contexts=(512,)),
    "cfg2": Workload("cfg2", "llama32_3b", 16, 16, 64, context_range=(128, 2048),
                     shared_prefix=1024, n_sharers=8),
    "cfg3": Workload("cfg3", "qwen3_8b", 16, 16, 64, contexts=(4096,) * 16),
    "cfg3_l4": Workload("cfg3_l4", "qwen3_8b_l4", 16, 16, 64, contexts=(4096,) * 16),
    "cfg4": Workload("cfg4", "qwen3_30b_a3b", 16, 16, 32, context_range=(256, 4096),
                     shared_prefix=2048, n_sharers=8),
    "cfg4_l4": Workload("cfg4_l4", "qwen3_30b_a3b_l4", 16, 16, 32, context_range=(256, 4096),
                        shared_prefix=2048, n_sharers=8),
    # one request alone on the larger dense shapes (the persistent kernel's wide classes)
    "b1_3b": Workload("b1_3b", "llama32_3b", 1, 16, 64, contexts=(512,)),
    "b1_8b": Workload("b1_8b", "qwen3_8b", 1, 16, 64, contexts=(512,)),
    "cfg0_q4": Workload("cfg0_q4", "tiny_q4", 5, 16, 6, contexts=(40, 16, 3, 0, 65)),
    "cfg0_moe": Workload("cfg0_moe", "tiny_moe", 3, 16, 4, contexts=(33, 16, 5)),
}
