"""Invariants that pin the oracle's method-level steps (tree, verify, accept, compact, draft).

 #1  a tree node's outputs equal a plain causal forward of (context + its root path)   [Sec. 3.4.1]
 #2  emitted tokens equal plain greedy autoregressive decoding                         [Sec. 4.1]
 #3  the acceptance walk equals an exhaustive search over root paths                   [Fig. 2, Sec. 3.4]
 #4  draft-after-accept (S1) and verify-and-draft-in-one-forward (S2) give the same drafts
 #5  pseudo rows fed with the *true* hidden states reproduce the true logits: pins the draft
     pass's positions, entry layers and mask                                            [Sec. 3.2, 3.3]
"""
import itertools

import numpy as np
import pytest

from ht_inputs import WORKLOADS, make_weights, prune_tree, random_tree, chain_tree, star_tree
from oracle import ht_oracle as O
from helpers import small_workload, oracle_model, oracle_decoder, prompt_of, tree_of


def _path(parent, v):
    p = []
    while v >= 0:
        p.append(v)
        v = parent[v]
    return p[::-1]


# ------------------------------------------------------------------ masks / depths by brute force
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_ancestor_matrix_and_depth_by_walking(seed):
    parent, _ = random_tree(seed, 40, 5)
    anc, depth = O.ancestor_matrix(parent), O.tree_depth(parent)
    for v in range(40):
        path = _path(parent, v)
        assert depth[v] == len(path) - 1 and anc[v].sum() == depth[v] + 1
        assert sorted(np.nonzero(anc[v])[0]) == sorted(path)


# ------------------------------------------------------------------ invariant 1, attention level
@pytest.mark.parametrize("maker", [lambda: random_tree(5, 24, 4), lambda: chain_tree(9), lambda: star_tree(9),
                                   lambda: ([-1], [0])])
def test_tree_attention_equals_causal_attention_over_each_path(maker):
    parent, _ = maker()
    t, n, hq, hkv, hd = len(parent), 11, 4, 2, 8
    rng = np.random.default_rng(7)
    q = rng.normal(size=(t, hq, hd))
    k_all, v_all = rng.normal(size=(n + t, hkv, hd)), rng.normal(size=(n + t, hkv, hd))
    depth, anc = O.tree_depth(parent), O.ancestor_matrix(parent)
    pos = np.array([n + e for e in depth])
    qr = O.rope(q, pos, 1e4)
    kr = O.rope(k_all, np.concatenate([np.arange(n), pos]), 1e4)
    vis = np.concatenate([np.ones((t, n), dtype=bool), anc], axis=1)
    got = O.masked_attention(qr, kr, v_all, vis)
    for v in range(t):
        path = _path(parent, v)
        rows = list(range(n)) + [n + u for u in path]
        # plain causal attention of the last token of the sequence (context ++ path): all keys visible,
        # keys at consecutive positions 0 .. n+depth
        kk = O.rope(k_all[rows], np.arange(len(rows)), 1e4)
        qq = O.rope(q[v:v + 1], np.array([len(rows) - 1]), 1e4)
        want = O.masked_attention(qq, kk, v_all[rows], np.ones((1, len(rows)), dtype=bool))
        assert np.allclose(got[v], want[0], atol=1e-12)


# ------------------------------------------------------------------ invariant 1, model level
@pytest.mark.parametrize("name", ["tiny", "tiny_k3", "tiny_full7"])
def test_verify_logits_equal_causal_forward_of_each_root_path(name):
    wl = WORKLOADS[name]
    model = oracle_model(wl)
    dec = oracle_decoder(wl, model)
    prompt = prompt_of(wl, 12)
    dec.prefill(prompt)
    rng = np.random.default_rng(0)
    tok = [dec.root] + [int(x) for x in rng.integers(0, wl.vocab, dec.T - 1)]
    z, g, saved = dec.verify(tok)
    _, hidden, ks, vs = model.causal_forward(prompt)                             # prefill == causal forward
    assert np.allclose(dec.K[1][:12], ks[1], atol=0)
    for v in range(dec.T):
        seq = prompt + [tok[u] for u in _path(dec.parent, v)]
        zz, hid, kk, _ = model.causal_forward(seq)
        assert np.max(np.abs(z[v] - zz[-1])) < 1e-9
        assert g[v] == int(np.argmax(zz[-1]))
        for t, h in saved.items():
            assert np.max(np.abs(h[v] - hid[t][-1])) < 1e-9
        assert np.max(np.abs(dec.K[1][dec.n + v] - kk[1][-1])) < 1e-9               # K written to slot n+v


# ------------------------------------------------------------------ invariant 2: losslessness
@pytest.mark.parametrize("name", ["tiny", "tiny_k3", "tiny_full7", "tiny_bf16"])
def test_sixteen_steps_equal_greedy_autoregressive(name):
    wl = WORKLOADS[name]
    model = oracle_model(wl)
    dec = oracle_decoder(wl, model)
    prompt = prompt_of(wl)
    dec.prefill(prompt)
    first_root = dec.root
    out = []
    for _ in range(16):
        res = dec.step()
        assert res["emitted"][0] == res["tok"][0]
        out += res["emitted"]
    want = model.ar_greedy(prompt, len(out) + 1)
    assert out[0] == first_root
    assert out == want[:len(out)] and dec.root == want[len(out)]
    assert dec.n == len(prompt) + len(out)
    # compaction: cache rows [0, n) are the K/V of a fresh causal forward of everything accepted
    _, hidden, ks, vs = model.causal_forward(prompt + out)
    for layer in range(wl.n_layers):
        assert np.max(np.abs(dec.K[layer][:dec.n] - ks[layer])) < 1e-9
        assert np.max(np.abs(dec.V[layer][:dec.n] - vs[layer])) < 1e-9
    for t, h in dec.h_src.items():
        assert np.max(np.abs(h - hidden[t][-1])) < 1e-9


def test_distinct_transfer_layers_are_lossless_too():
    wl = small_workload(n_layers=4, k=3, transfer_layers=(1, 2, 3), branching=(2, 2, 1), tree_size=8)
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    dec = oracle_decoder(wl, model)
    prompt = prompt_of(wl)
    dec.prefill(prompt)
    out = []
    for _ in range(6):
        out += dec.step()["emitted"]
    assert out == model.ar_greedy(prompt, len(out))


# ------------------------------------------------------------------ forced acceptance + invariant 3
def _forced_tokens(dec, truth, target_path, vocab):
    """Tokens that make exactly `target_path` (node ids from the root) acceptable."""
    wrong = [t for t in range(vocab) if t not in set(truth)]
    tok = [wrong[v] for v in range(dec.T)]
    for j, node in enumerate(target_path):
        tok[node] = truth[j]
    return tok


def _exhaustive_accept(parent, tok, g):
    """All root paths whose every non-root token equals the greedy choice after its parent; the longest."""
    t = len(parent)
    good = []
    for v in range(t):
        path = _path(parent, v)
        if all(tok[c] == g[p] for p, c in zip(path[:-1], path[1:])):
            good.append(path)
    best = max(len(p) for p in good)
    longest = [p for p in good if len(p) == best]
    return longest


@pytest.mark.parametrize("name", ["tiny", "tiny_k3"])
def test_forced_acceptance_every_prefix_of_every_root_path(name):
    wl = WORKLOADS[name]
    model = oracle_model(wl)
    prompt = prompt_of(wl, 10)
    truth = model.ar_greedy(prompt, wl.k + 3)                                      # truth[0] is the root
    probe = oracle_decoder(wl, model)
    seen = set()
    for leaf in range(probe.T):
        full = _path(probe.parent, leaf)
        for m_star in range(1, len(full) + 1):
            target = tuple(full[:m_star])
            if target in seen:
                continue
            seen.add(target)
            dec = oracle_decoder(wl, model)
            dec.prefill(prompt)
            assert dec.root == truth[0]
            tok = _forced_tokens(dec, truth, target, wl.vocab)
            res = dec.step(forced_tokens=tok)
            assert res["path"] == list(target) and len(res["emitted"]) == m_star
            assert res["emitted"] == truth[:m_star] and res["root"] == truth[m_star]
            longest = _exhaustive_accept(dec.parent, tok, res["g"])
            assert longest == [list(target)]                                        # unique and equal to the walk
            # and decoding simply continues correctly afterwards
            nxt = dec.step()
            assert nxt["emitted"][0] == truth[m_star]
    assert len(seen) == probe.T


def test_accept_walk_against_exhaustive_search_on_random_tiny_trees():
    rng = np.random.default_rng(4)
    for trial in range(300):
        t = int(rng.integers(1, 9))
        parent, _ = random_tree(int(rng.integers(1, 10 ** 6)), t, 3)
        # distinct tokens among siblings, tiny vocabulary so matches are common
        tok = [0] * t
        for p in range(t):
            kids = [c for c in range(t) if parent[c] == p]
            for c, x in zip(kids, rng.permutation(6)[:len(kids)]):
                tok[c] = int(x)
        g = [int(x) for x in rng.integers(0, 6, t)]
        path, nxt = O.accept_walk(parent, tok, g)
        longest = _exhaustive_accept(parent, tok, g)
        assert longest == [path] and nxt == g[path[-1]]


def test_duplicate_sibling_tokens_take_the_lowest_node_index():
    parent = [-1, 0, 0, 1, 2]
    path, nxt = O.accept_walk(parent, [9, 4, 4, 7, 7], [4, 7, 7, 1, 2])
    assert path == [0, 1, 3] and nxt == 1


# ------------------------------------------------------------------ invariant 5: draft semantics
@pytest.mark.parametrize("layers", [(1, 1), (1, 2), (2, 2), (1, 3)])
def test_draft_rows_fed_true_hidden_states_reproduce_true_logits(layers):
    wl = small_workload(n_layers=4, k=2, transfer_layers=layers)
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    seq = prompt_of(wl, 9)
    n = 7
    z, hidden, _, _ = model.causal_forward(seq)
    dec = oracle_decoder(wl, model)
    dec.prefill(seq[:n])
    # pseudo row i stands for the token at position n-1+i: feed it that token's real layer-t_i residual
    true_rows = [hidden[t][n - 1 + (i + 1)] for i, t in enumerate(layers)]
    d = dec.draft(true_rows)
    assert np.max(np.abs(d - z[n:n + 2])) < 1e-10
    # and a wrong position, or hiding row 1 from row 2, must break it (the pin has teeth)
    dec.n -= 1
    assert np.max(np.abs(dec.draft(true_rows) - z[n:n + 2])) > 1e-6


# ------------------------------------------------------------------ invariant 4: S1 == S2
@pytest.mark.parametrize("layers", [(1, 1), (1, 2)])
def test_fused_schedule_gives_the_same_drafts(layers):
    wl = small_workload(n_layers=3, k=2, transfer_layers=layers, d_model=16)
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    prompt = prompt_of(wl, 8)
    truth = model.ar_greedy(prompt, 4)
    for target in ([0], [0, 1], [0, 1, 3], [0, 2, 5]):
        s1, s2 = oracle_decoder(wl, model), oracle_decoder(wl, model)
        s1.prefill(prompt)
        s2.prefill(prompt)
        tok = _forced_tokens(s1, truth, target, wl.vocab)
        z2, g2, d_all = s2.fused_verify_and_draft(tok)
        res = s1.step(forced_tokens=tok)
        assert np.max(np.abs(res["Z"] - z2)) < 1e-10 and res["g"] == g2
        assert res["path"] == target
        d_next = s1.draft(s1.transfer())                                          # S1: draft after accepting
        assert np.max(np.abs(d_next - d_all[target[-1]])) < 1e-9
        assert np.std(d_next) > 1e-3
