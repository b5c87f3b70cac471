"""Stored values under tests/golden/.

`tree_mask_seven_nodes.txt` is typed by hand from the definition of tree attention (Sec. 3.4.1): the oracle's tree
tables have to reproduce it.  `dynamic_tree_two_levels.txt` is worked by hand from the product rule for independent
draws: the oracle's tree selection has to reproduce it.  `tiny_decode_trace.txt` is written by `tests/golden/make_golden.py` from the oracle
alone; the oracle has to keep reproducing it (a deliberate change regenerates the file and says why), and the GPU
test in test_gpu_parity.py decodes the same tokens through the C ABI.
"""
import os

import numpy as np

from ht_inputs import WORKLOADS
from oracle import ht_oracle as O
from helpers import oracle_decoder, oracle_model, prompt_of

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_tree_fixture():
    rows, mask, paths = {}, {}, {}
    for line in open(os.path.join(GOLDEN, "tree_mask_seven_nodes.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "mask":
            mask[int(f[1])] = [int(x) for x in f[2:]]
        elif f[0] == "path":
            paths[int(f[1])] = [int(x) for x in f[2:]]
        else:
            rows[f[0]] = [int(x) for x in f[1:]]
    return rows, mask, paths


def read_dynamic_tree_fixture():
    prob, trees = {}, {}
    for line in open(os.path.join(GOLDEN, "dynamic_tree_two_levels.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "prob":
            prob[int(f[1])] = [float(x) for x in f[2:]]
        else:
            trees.setdefault(int(f[1]), {})[f[2]] = [float(x) if f[2] == "reach" else int(x) for x in f[3:]]
    return prob, trees


def read_trace():
    """{workload: {"root": r, "steps": [{"tok": .., "path": .., "emitted": .., "next_root": .., "cache_len": ..}]}}"""
    out, cur = {}, None
    for line in open(os.path.join(GOLDEN, "tiny_decode_trace.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if f[0] == "workload":
            cur = out.setdefault(f[1], {"seed": int(f[3]), "prompt_len": int(f[5]), "tree_size": int(f[7]), "steps": []})
        elif f[0] == "root":
            cur["root"] = int(f[1])
        elif f[0] == "step":
            s = int(f[1])
            while len(cur["steps"]) <= s:
                cur["steps"].append({})
            if f[2] == "next_root":
                cur["steps"][s]["next_root"], cur["steps"][s]["cache_len"] = int(f[3]), int(f[5])
            else:
                cur["steps"][s][f[2]] = [int(x) for x in f[3:]]
    return out


def test_hand_written_tree_tables():
    rows, mask, paths = read_tree_fixture()
    parent, rank, depth = rows["parent"], rows["rank"], rows["depth"]
    T = len(parent)
    assert O.tree_depth(parent) == depth
    anc = O.ancestor_matrix(parent)
    assert anc.shape == (T, T)
    for v in range(T):
        assert [int(b) for b in anc[v]] == mask[v], f"mask row {v}"
    for v, path in paths.items():                       # the mask row of a leaf is its candidate sequence
        assert sorted(np.nonzero(anc[v])[0]) == path
    # the decoder derives the candidates per draft position from the ranks; a node's token is a function of
    # (depth, rank) only
    wl = WORKLOADS["tiny_k3"]
    dec = O.HiddenTransferOracle(oracle_model(wl), parent, rank, 64)
    assert dec.width[1:] == rows["width"]
    dec.root = 5
    cand = [[], [11, 12], [21, 22], [31]]
    assert dec.build_tree(cand) == [5, 11, 12, 21, 22, 21, 31]
    # greedy acceptance on it (Sec. 3.4): the walk follows children that carry the arg-max of their parent's row
    tok = dec.build_tree(cand)
    g = [11, 22, 0, 0, 7, 0, 0]                         # root -> 11 (node 1) -> 22 (node 4) -> 7 is nobody's token
    assert O.accept_walk(parent, tok, g) == ([0, 1, 4], 7)
    g = [12, 0, 21, 0, 0, 9, 0]                         # root -> 12 (node 2) -> 21 (node 5, not node 3) -> 9
    assert O.accept_walk(parent, tok, g) == ([0, 2, 5], 9)
    g = [99, 0, 0, 0, 0, 0, 0]                          # nothing matches: only the root is accepted
    assert O.accept_walk(parent, tok, g) == ([0], 99)


def test_oracle_reproduces_the_stored_decode_trace():
    trace = read_trace()
    assert set(trace) == {"tiny", "tiny_t123"}
    for name, want in trace.items():
        wl = WORKLOADS[name]
        assert (wl.seed, wl.tree_size) == (want["seed"], want["tree_size"])
        dec = oracle_decoder(wl, oracle_model(wl))
        prompt = prompt_of(wl)
        assert len(prompt) == want["prompt_len"]
        dec.prefill(prompt)
        assert dec.root == want["root"]
        for s, st in enumerate(want["steps"]):
            res = dec.step()
            assert res["tok"] == st["tok"], f"{name} step {s}: tree tokens"
            assert (res["path"], res["emitted"]) == (st["path"], st["emitted"]), f"{name} step {s}: acceptance"
            assert (res["root"], res["n"]) == (st["next_root"], st["cache_len"]), f"{name} step {s}: state"
        # every step emits at least the pending root, and the trace holds steps that accept drafts
        assert all(len(st["path"]) >= 1 for st in want["steps"])


def test_hand_worked_dynamic_tree():
    prob, trees = read_dynamic_tree_fixture()
    lp = np.log(np.array([prob[1], prob[2]]))
    for size, want in trees.items():
        for kind in (np.float64, np.float32):
            parent, rank = O.dynamic_tree(lp.astype(kind), size)
            assert parent == want["parent"] and rank == want["rank"], (size, kind)
        depth = O.tree_depth(parent)
        reach = [1.0]
        for v in range(1, size):
            reach.append(reach[parent[v]] * prob[depth[v]][rank[v]])
        assert abs(sum(reach[1:]) - want["reach"][0]) < 1e-12
