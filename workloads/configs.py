"""The round configurations this repository is measured and checked on: the five of the
benchmark contract plus the paper's other published settings (13B: 50 draft tokens; 70B: 48).

Shapes follow the model families the paper evaluates (Section 5, "Models") and
its hyper-parameters (Appendix A, "EAGLE-2": 60 draft tokens, depth 6, 10 nodes
expanded per layer for the 7B/8B models).  Values are synthetic: the paper's
datasets and trained weights are not used anywhere.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Tuple


@dataclass(frozen=True)
class RoundConfig:
    name: str
    index: int              # 1-based position in the list of configurations
    dtype: str              # "fp32" or "bf16": type of H, W, Q, K, V, O
    batch: int              # sequences, each with its own tree
    vocab: int              # V
    hidden: int             # Hd
    depth: int              # D: number of LM-head passes = deepest tree layer
    topk: int               # k: children kept per row and nodes expanded per layer
    n_tree: int             # N: rows of the flattened tree, root included
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_lo: int          # KV prefix length; lo == hi means a fixed length
    prefix_hi: int
    n_layers: int           # independent KV sets attended per round
    w_std: float            # std of the LM-head weights
    accept: str             # "greedy", "sample" or "mixed" (even b greedy, odd b sample)
    temperature: float
    seed: int

    @property
    def n_cand(self) -> int:
        """C = k + (D-1) k^2 candidate nodes produced by D passes."""
        return self.topk + (self.depth - 1) * self.topk * self.topk

    @property
    def n_draft_rows(self) -> int:
        """R = 1 + (D-1) k LM-head rows per round."""
        return 1 + (self.depth - 1) * self.topk

    def frontier_rows(self, d: int) -> int:
        return 1 if d == 0 else self.topk

    def scaled(self, **kw) -> "RoundConfig":
        return replace(self, **kw)


@dataclass(frozen=True)
class DraftLayerConfig:
    """Shape of the draft model's decoder layer (the models' own layer shape)."""
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    eps: float = 1e-5
    rope_theta: float = 10000.0


# decoder-layer shapes of the model families behind the round configurations
DRAFT_LAYERS = {
    "llama2_7b": DraftLayerConfig(32, 32, 128, 11008, 1e-5, 10000.0),
    "llama3_8b": DraftLayerConfig(32, 8, 128, 14336, 1e-5, 500000.0),
    "llama2_13b_m50": DraftLayerConfig(40, 40, 128, 13824, 1e-5, 10000.0),
    "llama2_70b_m48": DraftLayerConfig(64, 8, 128, 28672, 1e-5, 10000.0),
}

_BASE_SEED = 20240616 * 10

CONFIGS: Tuple[RoundConfig, ...] = (
    RoundConfig("tiny_fp32", 1, "fp32", 1, 1000, 256, 3, 4, 16, 4, 4, 64,
                128, 128, 1, 0.05, "greedy", 1.0, _BASE_SEED + 1),
    RoundConfig("llama2_7b", 2, "bf16", 1, 32000, 4096, 6, 10, 60, 32, 32, 128,
                2048, 2048, 1, 0.02, "greedy", 1.0, _BASE_SEED + 2),
    RoundConfig("llama3_8b", 3, "bf16", 1, 128256, 4096, 6, 10, 60, 32, 8, 128,
                4096, 4096, 1, 0.02, "sample", 1.0, _BASE_SEED + 3),
    RoundConfig("llama_70b_layer", 4, "bf16", 1, 32000, 8192, 8, 10, 80, 64, 8, 128,
                8192, 8192, 80, 0.02, "greedy", 1.0, _BASE_SEED + 4),
    RoundConfig("batched_serving", 5, "bf16", 16, 32000, 4096, 6, 10, 60, 32, 32, 128,
                512, 16384, 1, 0.02, "mixed", 1.0, _BASE_SEED + 5),
    # Appendix A: 50 draft tokens for the 13B models, 48 for the 70B models (depth 6, 10 nodes per layer)
    RoundConfig("llama2_13b_m50", 6, "bf16", 1, 32000, 5120, 6, 10, 50, 40, 40, 128,
                2048, 2048, 1, 0.02, "greedy", 1.0, _BASE_SEED + 6),
    RoundConfig("llama2_70b_m48", 7, "bf16", 1, 32000, 8192, 6, 10, 48, 64, 8, 128,
                4096, 4096, 1, 0.02, "sample", 1.0, _BASE_SEED + 7),
)


def get_config(index_or_name) -> RoundConfig:
    for c in CONFIGS:
        if c.index == index_or_name or c.name == index_or_name:
            return c
    raise KeyError(index_or_name)
