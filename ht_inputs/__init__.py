"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package holds input *generators* only (weights, token ids, tree topologies, the named
workload shapes).  It contains none of the decoding method's arithmetic and imports neither
the oracle nor the HIP binding.
"""
from .generators import (  # noqa: F401
    counter_normal,
    counter_tokens,
    counter_u64_reference,
    make_weights,
    layer_weights,
    TENSOR_IDS,
)
from .trees import prune_tree, random_tree, chain_tree, star_tree, tree_depths  # noqa: F401
from .workloads import WORKLOADS, Workload  # noqa: F401
