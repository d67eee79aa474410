"""Shape/config record used by the oracle (test infrastructure, see package docstring)."""
from dataclasses import dataclass, field
from typing import Tuple

LORA_TARGETS = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass
class StageConfig:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int = 0
    n_experts: int = 0
    top_k: int = 0
    rope_base: float = 1.0e6
    rms_eps: float = 1.0e-6
    qk_norm: bool = True
    lora_rank: int = 0
    lora_scale: float = 1.0
    lora_targets: Tuple[str, ...] = field(default_factory=tuple)
    train_base: bool = True
    moe_router: bool = False   # MoE: the layer holds the router Wr [E, h]; logits = n2 Wr^T instead of being an input

    @property
    def qd(self):
        return self.n_q_heads * self.head_dim

    @property
    def kd(self):
        return self.n_kv_heads * self.head_dim

    def has_lora(self, name):
        return self.lora_rank > 0 and name in self.lora_targets
