"""The five verification workloads (shapes only)."""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class VerifyConfig:
    name: str
    dtype: str          # "f32" | "bf16": type of q/k/v and the cache
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_len: int         # prefix length per sequence and layer
    n_nodes: int        # draft-tree nodes, root included
    tree_depth: int
    tree_topk: int
    vocab: int
    accept: str         # "greedy" | "sample" (bench default; tests run both where stated)
    temperature: float = 1.0

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def attn_bytes_per_layer(self) -> int:
        """Algorithmic bytes of one attention launch: K and V of prefix and tree read once
        per kv head, Q read once and the output written once."""
        kv = 2 * (self.kv_len + self.n_nodes) * self.n_kv_heads * self.head_dim * self.itemsize
        qo = 2 * self.n_nodes * self.n_q_heads * self.head_dim * self.itemsize
        return self.batch * (kv + qo)

    def attn_flops_per_layer(self) -> int:
        """QK^T and PV at the true node count, 2 flops per multiply-add, mask not subtracted."""
        return self.batch * 4 * self.n_nodes * (self.kv_len + self.n_nodes) * self.n_q_heads * self.head_dim

    def logit_bytes(self) -> int:
        return self.batch * self.n_nodes * self.vocab * 4

    def step_bytes(self) -> int:
        return self.layers * self.attn_bytes_per_layer() + self.logit_bytes()

    def step_flops(self) -> int:
        return self.layers * self.attn_flops_per_layer()


CONFIGS = {
    # tiny fp32 parity case: the oracle finishes in well under a second
    "c0": VerifyConfig("c0-tiny-f32", "f32", 1, 1, 8, 8, 64, 256, 26, 5, 4, 1000, "greedy"),
    # Vicuna-7B-shaped layer
    "c1": VerifyConfig("c1-vicuna7b-layer", "bf16", 1, 1, 32, 32, 128, 2048, 26, 6, 4, 32000, "greedy"),
    # LLaMA3-8B-shaped GQA layer
    "c2": VerifyConfig("c2-llama3-8b-layer", "bf16", 1, 1, 32, 8, 128, 4096, 60, 6, 10, 128256, "sample"),
    # Vicuna-33B-shaped layer stack, 4 sequences with different trees
    "c3": VerifyConfig("c3-vicuna33b-stack", "bf16", 60, 4, 52, 52, 128, 4096, 60, 6, 10, 32000, "greedy"),
    # LLaMA3-70B-shaped long-context layer stack
    "c4": VerifyConfig("c4-llama3-70b-stack", "bf16", 80, 1, 64, 8, 128, 16384, 60, 6, 10, 128256, "sample"),
}
