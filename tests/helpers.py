"""Glue shared by the tests: build oracle objects from a named workload."""
from __future__ import annotations

import numpy as np
import torch

from ht_inputs import WORKLOADS, Workload, make_weights, counter_tokens, prune_tree
from ht_inputs.generators import PROMPT_STREAM
from oracle.ht_oracle import OracleConfig, OracleWeights, OracleModel, HiddenTransferOracle


def torch_dtype(wl: Workload):
    return torch.float32 if wl.dtype == "f32" else torch.bfloat16


def oracle_config(wl: Workload) -> OracleConfig:
    return OracleConfig(wl.n_layers, wl.d_model, wl.n_heads, wl.n_kv_heads, wl.head_dim, wl.d_ffn, wl.vocab,
                        wl.k, tuple(wl.transfer_layers), wl.rms_eps, wl.rope_base)


def oracle_model(wl: Workload, tensors=None) -> OracleModel:
    if tensors is None:
        tensors = make_weights(wl, wl.seed, "cpu", torch_dtype(wl))
    return OracleModel(oracle_config(wl), OracleWeights(tensors))


def prompt_of(wl: Workload, length=None):
    return [int(t) for t in counter_tokens(wl.seed, PROMPT_STREAM, length or wl.prompt_len, wl.vocab)]


def tree_of(wl: Workload):
    return prune_tree(wl.branching, wl.tree_size)


def oracle_decoder(wl: Workload, model=None, tree=None, capacity=None) -> HiddenTransferOracle:
    model = model or oracle_model(wl)
    parent, rank = tree or tree_of(wl)
    return HiddenTransferOracle(model, parent, rank, capacity or wl.max_cache)


def small_workload(**kw) -> Workload:
    """A shrunken model for loop-level brute force (seconds in pure Python)."""
    base = dict(name="mini", n_layers=2, d_model=16, n_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24, vocab=40,
                k=2, transfer_layers=(1, 1), dtype="f32", prompt_len=6, max_cache=48, tree_size=7,
                branching=(2, 2), seed=99)
    base.update(kw)
    return Workload(**base)
