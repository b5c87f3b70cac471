"""Named workload shapes (sizes only; no arithmetic)."""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    k: int                              # number of hidden-transfer steps (pseudo positions)
    transfer_layers: Tuple[int, ...]    # t_i: residual stream after t_i blocks (1-based block count)
    dtype: str                          # "f32" | "bf16"
    prompt_len: int
    max_cache: int
    tree_size: int                      # T, root included
    branching: Tuple[int, ...]
    seed: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


_SEED = 20240412

WORKLOADS: Dict[str, Workload] = {
    # tiny fp32 end-to-end model: k=2, 8-node tree over three levels (root, depth 1, depth 2)
    "tiny": Workload("tiny", 2, 256, 4, 4, 64, 688, 1024, 2, (1, 1), "f32", 32, 128, 8, (2, 2), _SEED + 0),
    # literal "top-2/top-2/top-1, depth 3" variant with three maps
    "tiny_k3": Workload("tiny_k3", 2, 256, 4, 4, 64, 688, 1024, 3, (1, 1, 1), "f32", 32, 128, 8, (2, 2, 1), _SEED + 0),
    # full [2,2] tree, odd node count
    "tiny_full7": Workload("tiny_full7", 2, 256, 4, 4, 64, 688, 1024, 2, (1, 1), "f32", 32, 128, 7, (2, 2), _SEED + 0),
    # tiny bf16 twin of "tiny" (GPU bf16 kernels at a size the oracle finishes instantly)
    "tiny_bf16": Workload("tiny_bf16", 2, 256, 4, 4, 64, 688, 1024, 2, (1, 1), "bf16", 32, 128, 8, (2, 2), _SEED + 0),
    # a different transfer layer for every step (Sec. 4.1), and two steps sharing one
    "tiny_t123": Workload("tiny_t123", 4, 256, 4, 4, 64, 688, 1024, 3, (1, 2, 3), "f32", 32, 128, 8, (2, 2, 1), _SEED + 0),
    "tiny_t112": Workload("tiny_t112", 3, 256, 4, 4, 64, 688, 1024, 3, (1, 1, 2), "f32", 32, 128, 8, (2, 2, 1), _SEED + 0),
    "tiny_t123_bf16": Workload("tiny_t123_bf16", 4, 256, 4, 4, 64, 688, 1024, 3, (1, 2, 3), "bf16", 32, 128, 8, (2, 2, 1),
                               _SEED + 0),
    "llama7b": Workload("llama7b", 32, 4096, 32, 32, 128, 11008, 32000, 3, (24, 24, 24), "bf16", 512, 1024, 64,
                        (10, 3, 2), _SEED + 2),
    "llama13b": Workload("llama13b", 40, 5120, 40, 40, 128, 13824, 32000, 3, (30, 30, 30), "bf16", 2048, 2560, 64,
                         (10, 3, 2), _SEED + 3),
    # the layers the paper's main experiments name (25 / 30 / 35 of 40, Sec. 4.1)
    "llama13b_t253035": Workload("llama13b_t253035", 40, 5120, 40, 40, 128, 13824, 32000, 3, (25, 30, 35), "bf16", 2048,
                                 2560, 64, (10, 3, 2), _SEED + 3),
    "llama70b": Workload("llama70b", 80, 8192, 64, 8, 128, 28672, 32000, 4, (60, 60, 60, 60), "bf16", 4096, 4608, 64,
                         (10, 3, 2, 2), _SEED + 4),
}

# tree-attention op alone: 32 heads x 128, cache 4096, random 128-node tree of depth <= 6
ATTENTION_OP = dict(n_heads=32, n_kv_heads=32, head_dim=128, cache_len=4096, tree_size=128, max_depth=6,
                    rope_base=10000.0, seed=_SEED + 1)
