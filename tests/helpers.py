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


class WidenedOnRead:
    """Stored matrices (one per layer) that are handed out as fp64 copies, made when an entry is read and kept only
    until another entry is read: the oracle then runs a model whose fp64 copy would not fit the host memory, with its
    arithmetic untouched (it reads `w.wq[layer]` and gets the same fp64 matrix as from an `OracleWeights`)."""

    def __init__(self, stored):
        self.stored, self.at, self.wide = list(stored), None, None

    def __len__(self):
        return len(self.stored)

    def __getitem__(self, layer):
        if self.at != layer:
            self.wide = None
            self.wide = self.stored[layer].detach().to("cpu").double().numpy()
            self.at = layer
        return self.wide


def layerwise_oracle_model(wl: Workload, tensors) -> OracleModel:
    """`oracle_model` for a model too large to widen at once: the seven projections of a block are widened to fp64
    when the oracle reaches that block; embedding, head, gains and transfer maps are widened up front."""
    small = {k: v for k, v in tensors.items()}
    heavy = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
    for name in heavy:
        small[name] = []
    w = OracleWeights(small)
    for name in heavy:
        setattr(w, name, WidenedOnRead(tensors[name]))
    return OracleModel(oracle_config(wl), w)


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
