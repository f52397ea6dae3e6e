"""The five seeded synthetic configurations (shapes only, no arithmetic).

Each entry fixes one MoE layer shape in the notation of the paper's
preliminaries (Sec. 3.1: N_r routed experts, Top-K routing, per-layer cache
capacity C) plus the input recipe.  The shapes are those of DeepSeek-V2-Lite,
Qwen1.5-MoE-A2.7B and Qwen3-30B-A3B; hidden states and weights are synthetic.
"""
from dataclasses import dataclass, field
from typing import Tuple


@dataclass(frozen=True)
class MoEConfig:
    name: str
    n_layers: int          # L
    hidden: int            # H
    n_experts: int         # N_r
    inter: int             # I   (routed expert intermediate size)
    top_k: int             # K
    renorm: bool           # renormalise the K selected probabilities
    shared_inter: int      # I_s (total shared intermediate, 0 = none)
    shared_gate: bool      # shared expert scaled by sigmoid(w.x)
    dtype: str             # "f32" or "bf16": x, expert weights, y
    n_seq: int             # S
    seq_len: int           # T_s
    rhos: Tuple[float, ...]            # AR(1) correlation(s) of the hidden states
    capacities: Tuple[int, ...]        # LRU capacity C (experts per layer)
    seed: int
    decode: bool = False   # M=1 sequential decode steps instead of a batched forward
    weight_std: float = 0.02

    @property
    def n_tokens(self) -> int:
        return self.n_seq * self.seq_len

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def expert_bytes(self) -> int:
        """Bytes of one routed expert's three matrices (gate, up, down)."""
        return 3 * self.hidden * self.inter * self.elem_bytes

    @property
    def flops_per_token_layer(self) -> int:
        """Algorithmic flops of one token through one layer: router, K routed
        SwiGLU experts and the shared expert (multiply-add = 2 flops)."""
        h = self.hidden
        return (2 * h * self.n_experts + 6 * self.top_k * h * self.inter
                + 6 * h * self.shared_inter + (2 * h if self.shared_gate else 0))

    @property
    def decode_bytes_per_layer_step(self) -> int:
        """Algorithmic HBM bytes of one M=1 layer step: fp32 router matrix, the K
        selected experts' weights, and the x / y vectors."""
        h = self.hidden
        return (self.n_experts * h * 4 + self.top_k * self.expert_bytes
                + 3 * h * self.shared_inter * self.elem_bytes + 2 * h * self.elem_bytes)


CONFIGS = {
    "tiny": MoEConfig("tiny", 1, 256, 16, 128, 2, False, 0, False, "f32",
                      1, 128, (0.8,), (4,), 0),
    "dsv2lite": MoEConfig("dsv2lite", 4, 2048, 64, 1408, 6, False, 2816, False, "bf16",
                          8, 2048, (0.8,), (16,), 1),
    "qwen15moe": MoEConfig("qwen15moe", 8, 2048, 60, 1408, 4, False, 5632, True, "bf16",
                           64, 1024, (0.0, 0.8), (12,), 2),
    "qwen3_prefill": MoEConfig("qwen3_prefill", 48, 2048, 128, 768, 8, True, 0, False, "bf16",
                               16, 4096, (0.8,), (32,), 3),
    "qwen3_decode": MoEConfig("qwen3_decode", 48, 2048, 128, 768, 8, True, 0, False, "bf16",
                              1, 4096, (0.0, 0.5, 0.9), (16, 32, 64), 4, decode=True),
}


def get_config(name: str) -> MoEConfig:
    return CONFIGS[name]
