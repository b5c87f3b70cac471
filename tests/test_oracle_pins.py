"""Pins for the CPU oracle: closed forms, loop-level brute force and special cases.

No value in the paper fixes a float, so the oracle's arithmetic is pinned to mathematics instead:
each primitive against a closed form or a scalar-loop evaluation written independently here, and
the block against a pure-Python scalar transformer on a very small model.
"""
import math

import numpy as np
import pytest
import torch

from ht_inputs import make_weights, counter_normal, counter_u64_reference, counter_tokens, prune_tree, \
    random_tree, tree_depths
from ht_inputs.generators import counter_token_reference
from oracle import ht_oracle as O
from helpers import small_workload, oracle_model, oracle_config


# ------------------------------------------------------------------ input generators (host side)
def test_counter_generator_matches_python_integers():
    t = counter_normal(11, 1003, (7, 9), 0.02)
    for i in (0, 1, 8, 9, 62):
        s = counter_u64_reference(11, 1003, i)
        want = np.float32(np.float32(s - 393210) / np.float32(65536.0)) * np.float32(0.02)
        assert t.view(-1)[i].item() == want
    g = counter_normal(11, 2, (64,), 0.02, mean=1.0)
    s = counter_u64_reference(11, 2, 5)
    want = np.float32(np.float32((s - 393210) / 65536.0) * np.float32(0.02)) + np.float32(1.0)
    assert g[5].item() == want


def test_counter_generator_chunking_and_moments():
    a = counter_normal(3, 5, (1000, 37), 1.0, chunk=1 << 24)
    b = counter_normal(3, 5, (1000, 37), 1.0, chunk=4099)
    assert torch.equal(a, b)
    assert abs(a.mean().item()) < 0.02 and abs(a.std().item() - 1.0) < 0.02
    toks = counter_tokens(3, 7, 50, 1024)
    assert [int(x) for x in toks] == [counter_token_reference(3, 7, i, 1024) for i in range(50)]
    assert toks.min() >= 0 and toks.max() < 1024


def test_prune_tree_shapes():
    for br, size, levels in [((10, 3, 2), 64, [1, 10, 21, 32]), ((10, 3, 2), 16, [1, 4, 5, 6]),
                             ((10, 3, 2), 32, [1, 6, 11, 14]), ((2, 2), 8, [1, 3, 4]), ((2, 2), 7, [1, 2, 4]),
                             ((2, 2, 1), 8, [1, 2, 3, 2]), ((10, 3, 2), 1, [1])]:
        parent, rank = prune_tree(br, size)
        depth = tree_depths(parent)
        assert [depth.count(e) for e in range(max(depth) + 1)] == levels
        assert parent[0] == -1 and all(0 <= parent[v] < v for v in range(1, size))
        sib = {(parent[v], rank[v]) for v in range(1, size)}
        assert len(sib) == size - 1                      # distinct rank among siblings
        for v in range(1, size):                          # rank-closed: a rank-r child implies rank r-1 sibling
            assert rank[v] == 0 or (parent[v], rank[v] - 1) in sib


# ------------------------------------------------------------------ primitives: closed forms
def test_rms_norm_closed_forms():
    g = np.array([2.0, -1.0])
    out = O.rms_norm(np.array([[3.0, 4.0]]), g, 0.0)
    assert np.allclose(out, [[3.0 / math.sqrt(12.5) * 2.0, -4.0 / math.sqrt(12.5)]], rtol=0, atol=1e-15)
    c = np.full((1, 8), 0.5)
    assert np.allclose(O.rms_norm(c, np.ones(8), 1e-5), 0.5 / math.sqrt(0.25 + 1e-5), atol=1e-15)
    x = np.random.default_rng(0).normal(size=(3, 32))
    y = O.rms_norm(x, np.ones(32), 0.0)
    assert np.allclose((y * y).mean(axis=1), 1.0, atol=1e-12)
    assert np.allclose(O.rms_norm(7.0 * x, np.ones(32), 0.0), y, atol=1e-12)       # scale invariant when eps = 0


def test_rope_closed_forms():
    # hd = 2: one pair, frequency base^0 = 1, so position p is a plain rotation by p radians
    x = np.array([[[1.0, 0.0]], [[0.3, -0.7]]])
    out = O.rope(x, np.array([2, 5]), 10000.0)
    assert np.allclose(out[0, 0], [math.cos(2.0), math.sin(2.0)], atol=1e-15)
    assert np.allclose(out[1, 0], [0.3 * math.cos(5) + 0.7 * math.sin(5), -0.7 * math.cos(5) + 0.3 * math.sin(5)],
                       atol=1e-15)
    # hd = 4: pairs (0,2) and (1,3); second pair turns at base^(-2/4)
    y = O.rope(np.array([[[1.0, 1.0, 0.0, 0.0]]]), np.array([3]), 100.0)
    assert np.allclose(y[0, 0], [math.cos(3.0), math.cos(0.3), math.sin(3.0), math.sin(0.3)], atol=1e-15)
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=(1, 2, 16)), rng.normal(size=(1, 2, 16))
    assert np.allclose(O.rope(q, np.array([0]), 10000.0), q, atol=0)                # position 0 is the identity
    assert np.allclose(np.linalg.norm(O.rope(q, np.array([17]), 10000.0)), np.linalg.norm(q), atol=1e-12)
    dots = [np.sum(O.rope(q, np.array([a]), 1e4) * O.rope(k, np.array([a - 4]), 1e4), axis=-1) for a in (4, 9, 300)]
    assert np.allclose(dots[0], dots[1], atol=1e-12) and np.allclose(dots[0], dots[2], atol=1e-11)


def test_silu_closed_forms():
    x = np.array([-30.0, -1.0, 0.0, 1.0, 30.0])
    s = O.silu(x)
    assert s[2] == 0.0 and np.allclose(s - O.silu(-x), x, atol=1e-12)
    assert abs(s[3] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15 and abs(s[4] - 30.0) < 1e-10


def _attention_loops(q, keys, values, visible):
    r, hq, hd = q.shape
    group = hq // keys.shape[1]
    out = np.zeros_like(q)
    for a in range(r):
        for h in range(hq):
            js = [j for j in range(keys.shape[0]) if visible[a][j]]
            sc = [sum(q[a, h, e] * keys[j, h // group, e] for e in range(hd)) / math.sqrt(hd) for j in js]
            mx = max(sc)
            w = [math.exp(s - mx) for s in sc]
            tot = sum(w)
            for e in range(hd):
                out[a, h, e] = sum(wj * values[j, h // group, e] for wj, j in zip(w, js)) / tot
    return out


def test_masked_attention_against_loops_and_limits():
    rng = np.random.default_rng(2)
    q, keys, vals = rng.normal(size=(5, 4, 6)), rng.normal(size=(9, 2, 6)), rng.normal(size=(9, 2, 6))
    vis = rng.random((5, 9)) < 0.6
    vis[:, 0] = True
    assert np.allclose(O.masked_attention(q, keys, vals, vis), _attention_loops(q, keys, vals, vis), atol=1e-13)
    # q = 0 -> uniform weights -> mean of the visible values (GQA: head h reads kv head h // 2)
    out = O.masked_attention(np.zeros_like(q), keys, vals, vis)
    for a in range(5):
        for h in range(4):
            assert np.allclose(out[a, h], vals[vis[a], h // 2].mean(axis=0), atol=1e-13)
    one = np.zeros((5, 9), dtype=bool)
    one[np.arange(5), [3, 1, 4, 1, 5]] = True                                      # a single visible key
    out = O.masked_attention(q, keys, vals, one)
    assert np.allclose(out[2, 3], vals[4, 1], atol=1e-13)


def test_top_candidates_order_and_ties():
    row = np.array([0.5, 2.0, 2.0, -1.0, 2.0, 0.5, 3.0])
    assert O.top_candidates(row, 5) == [6, 1, 2, 4, 0]
    rng = np.random.default_rng(3)
    r = np.round(rng.normal(size=200), 1)                                           # many exact ties
    want = sorted(range(200), key=lambda j: (-r[j], j))[:17]
    assert O.top_candidates(r, 17) == want
    assert O.top_candidates(r, 1)[0] == int(np.argmax(r))                           # argmax tie -> lowest id


# ------------------------------------------------------------------ whole block vs scalar Python
def _scalar_forward(cfg, w, tokens):
    """Pure-Python scalar causal transformer (independent of the numpy code path)."""
    L, d, hq, hkv, hd, f = cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn
    n = len(tokens)
    xs = [[float(w.tok_emb[t][c]) for c in range(d)] for t in tokens]

    def matvec(mat, vec):
        return [sum(float(mat[o][i]) * vec[i] for i in range(len(vec))) for o in range(len(mat))]

    def norm(vec, gain):
        ms = sum(a * a for a in vec) / len(vec)
        return [a / math.sqrt(ms + cfg.rms_eps) * float(gg) for a, gg in zip(vec, gain)]

    def rot(vec, p):
        out = list(vec)
        for h in range(len(vec) // hd):
            for j in range(hd // 2):
                ang = p * cfg.rope_base ** (-2.0 * j / hd)
                a, b = vec[h * hd + j], vec[h * hd + j + hd // 2]
                out[h * hd + j] = a * math.cos(ang) - b * math.sin(ang)
                out[h * hd + j + hd // 2] = b * math.cos(ang) + a * math.sin(ang)
        return out

    for layer in range(L):
        us = [norm(x, w.attn_norm[layer]) for x in xs]
        qs = [rot(matvec(w.wq[layer], u), p) for p, u in enumerate(us)]
        ks = [rot(matvec(w.wk[layer], u), p) for p, u in enumerate(us)]
        vs = [matvec(w.wv[layer], u) for u in us]
        new = []
        for p in range(n):
            att = []
            for h in range(hq):
                g = h // (hq // hkv)
                sc = [sum(qs[p][h * hd + e] * ks[j][g * hd + e] for e in range(hd)) / math.sqrt(hd) for j in range(p + 1)]
                mx = max(sc)
                ex = [math.exp(s - mx) for s in sc]
                tot = sum(ex)
                att += [sum(ex[j] * vs[j][g * hd + e] for j in range(p + 1)) / tot for e in range(hd)]
            x = [a + b for a, b in zip(xs[p], matvec(w.wo[layer], att))]
            u2 = norm(x, w.ffn_norm[layer])
            gate, up = matvec(w.w_gate[layer], u2), matvec(w.w_up[layer], u2)
            act = [gg / (1.0 + math.exp(-gg)) * uu for gg, uu in zip(gate, up)]
            new.append([a + b for a, b in zip(x, matvec(w.w_down[layer], act))])
        xs = new
    return [matvec(w.lm_head, norm(x, w.final_norm)) for x in xs]


def test_causal_forward_against_scalar_python():
    wl = small_workload()
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    tokens = [3, 17, 5, 39, 0, 22, 8]
    z, hidden, ks, vs = model.causal_forward(tokens)
    want = np.array(_scalar_forward(model.cfg, model.w, tokens))
    assert np.max(np.abs(z - want)) < 1e-11
    assert np.std(want) > 0.05                                                     # not a vacuous comparison


def test_causality_and_degenerate_blocks():
    wl = small_workload()
    tensors = make_weights(wl, wl.seed, sigma=0.4)
    model = oracle_model(wl, tensors)
    a, _, _, _ = model.causal_forward([1, 2, 3, 4, 5])
    b, _, _, _ = model.causal_forward([1, 2, 3, 9, 7])
    assert np.allclose(a[:3], b[:3], atol=1e-13) and not np.allclose(a[3], b[3])
    # zero output projections switch both sub-layers off: logits = rms(E[tok]) @ W_lm^T
    for layer in range(wl.n_layers):
        tensors["wo"][layer] = torch.zeros_like(tensors["wo"][layer])
        tensors["w_down"][layer] = torch.zeros_like(tensors["w_down"][layer])
    off = oracle_model(wl, tensors)
    z, _, _, _ = off.causal_forward([4, 4, 11])
    e = off.w.tok_emb[[4, 4, 11]]
    want = (e / np.sqrt((e * e).mean(axis=1, keepdims=True) + wl.rms_eps) * off.w.final_norm) @ off.w.lm_head.T
    assert np.allclose(z, want, atol=1e-14) and np.allclose(z[0], z[1], atol=0)


def test_transfer_is_a_bare_matrix_product():
    wl = small_workload(k=3, transfer_layers=(1, 1, 2), n_layers=3)
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    dec = O.HiddenTransferOracle(model, [-1, 0], [0, 0], 32)
    prompt = [5, 6, 7, 8]
    dec.prefill(prompt)
    _, hidden, _, _ = model.causal_forward(prompt)
    ps = dec.transfer()
    for i, t in enumerate(wl.transfer_layers):
        h = hidden[t][-1]
        want = [sum(model.w.w_transfer[i][o, c] * h[c] for c in range(wl.d_model)) for o in range(wl.d_model)]
        assert np.allclose(ps[i], want, atol=1e-13)


# ------------------------------------------------------------------ tree chosen from the draft distributions
def test_candidate_logprobs_closed_forms():
    from scipy.special import log_softmax
    V = 37
    ids, lp = O.candidate_logprobs(np.full(V, 3.25), 5)
    assert ids == [0, 1, 2, 3, 4]                                  # equal values: lowest ids first
    assert np.allclose(lp, -math.log(V), atol=1e-13)               # uniform distribution
    rng = np.random.default_rng(5)
    z = rng.normal(size=V) * 4
    ids, lp = O.candidate_logprobs(z, V)
    assert sorted(ids) == list(range(V)) and np.all(np.diff(lp) <= 0)
    assert abs(np.sum(np.exp(lp)) - 1.0) < 1e-13                   # the whole vocabulary: a distribution
    ids7, lp7 = O.candidate_logprobs(z, 7)
    assert ids7 == ids[:7] and np.array_equal(lp7, lp[:7])
    assert np.allclose(lp7, log_softmax(z)[ids7], atol=1e-13)      # library routine at the same tokens
    _, shifted = O.candidate_logprobs(z + 1000.0, 7)               # softmax ignores a common shift
    assert np.allclose(shifted, lp7, atol=1e-10)
    two = np.array([0.0, math.log(3.0)])                           # probabilities 1/4 and 3/4
    ids, lp = O.candidate_logprobs(two, 2)
    assert ids == [1, 0] and np.allclose(np.exp(lp), [0.75, 0.25], atol=1e-15)


def _all_nodes(k, b):
    import itertools
    return [p for e in range(1, k + 1) for p in itertools.product(range(b), repeat=e)]


@pytest.mark.parametrize("k,b,sizes", [(2, 2, range(1, 8)), (2, 3, range(1, 8)), (3, 2, range(1, 8)), (3, 3, range(1, 6))])
def test_dynamic_tree_is_the_best_tree_of_its_size(k, b, sizes):
    """Exhaustive search: among all parent-closed node sets of the same size none is reached more often."""
    import itertools
    rng = np.random.default_rng(100 * k + b)
    for trial in range(3):
        lp = np.stack([O.candidate_logprobs(rng.normal(size=3 * b + trial) * 2, b)[1] for _ in range(k)])
        nodes = _all_nodes(k, b)
        reach = {p: math.exp(sum(lp[e, r] for e, r in enumerate(p))) for p in nodes}
        for T in sizes:
            parent, rank = O.dynamic_tree(lp, T)
            assert len(parent) == T and parent[0] == -1
            assert all(0 <= parent[v] < v for v in range(1, T))
            paths = [()]
            for v in range(1, T):
                paths.append(paths[parent[v]] + (rank[v],))
            assert len(set(paths)) == T                            # distinct nodes
            got = sum(reach[p] for p in paths[1:])
            best = 0.0
            for pick in itertools.combinations(nodes, T - 1):
                chosen = set(pick)
                if all(len(p) == 1 or p[:-1] in chosen for p in pick):
                    best = max(best, sum(reach[p] for p in pick))
            assert abs(got - best) <= 1e-12 * max(best, 1.0), (k, b, T, got, best)


def test_dynamic_tree_order_on_ties_and_degenerate_distributions():
    flat = np.full((2, 2), -1.0)                                   # all equal: level by level, paths in order
    assert O.dynamic_tree(flat, 7) == ([-1, 0, 0, 1, 1, 2, 2], [0, 0, 1, 0, 1, 0, 1])
    assert O.dynamic_tree(flat, 4) == ([-1, 0, 0, 1], [0, 0, 1, 0])
    assert O.dynamic_tree(flat, 1) == ([-1], [0])
    sure = np.array([[0.0, -np.inf, -np.inf]] * 3)                 # one certain token per position: the chain first,
    parent, rank = O.dynamic_tree(sure, 7)                         # then impossible nodes by depth and path
    assert parent == [-1, 0, 1, 2, 0, 0, 1] and rank == [0, 0, 0, 0, 1, 2, 1]
    nan = np.array([[-0.1, np.nan], [-0.2, -0.3]])                 # NaN counts as -inf
    assert O.dynamic_tree(nan, 5) == ([-1, 0, 1, 1, 0], [0, 0, 0, 1, 1])
    with pytest.raises(ValueError):
        O.dynamic_tree(flat, 8)                                    # 2 + 4 nodes below the root at most
    # a strictly better second level beats a worse first-level sibling: depth is only a tie-break
    lp = np.log(np.array([[0.9, 0.05], [0.8, 0.1]]))
    assert O.dynamic_tree(lp, 4) == ([-1, 0, 1, 1], [0, 0, 0, 1])  # 0.9, 0.72, 0.09 before 0.05


def test_dynamic_tree_decides_in_the_precision_of_its_input():
    c = -(0.5 - 2.0 ** -25)                                        # -0.5 + c = -(1 - 2^-25): rounds to -1 in float32
    lp32 = np.array([[-0.5, -1.0], [c, -10.0]], dtype=np.float32)
    assert float(lp32[1, 0]) == c
    assert O.dynamic_tree(lp32, 3) == ([-1, 0, 0], [0, 0, 1])      # float32: a tie, the shallower node first
    assert O.dynamic_tree(lp32.astype(np.float64), 3) == ([-1, 0, 1], [0, 0, 0])   # float64: the child is ahead


def test_oracle_step_with_a_dynamic_tree_stays_lossless():
    """Whatever tree a step picks, the emitted tokens are the greedy continuation (Sec. 4.1)."""
    wl = small_workload(k=2, transfer_layers=(1, 1), max_cache=64)
    model = oracle_model(wl)
    dec = O.HiddenTransferOracle(model, [-1], [0], wl.max_cache)
    prompt = [int(t) for t in counter_tokens(wl.seed, 1, wl.prompt_len, wl.vocab)]
    dec.prefill(prompt)
    out, shapes = [], set()
    for _ in range(6):
        res = dec.step(dynamic=(6, 3))
        assert len(dec.parent) == 6
        shapes.add(tuple(dec.parent))
        out += res["emitted"]
    want = model.ar_greedy(prompt, len(out))
    assert out == want[:len(out)]
    assert len(shapes) > 1                                         # the tree really changes between steps


# ------------------------------------------------------------------ training-stage forward (Sec. 3.3)
def test_kl_divergence_closed_forms_and_argument_order():
    a, b = np.log(np.array([0.75, 0.25])), np.log(np.array([0.5, 0.5]))
    assert abs(O.kl_divergence(a, b) - (0.75 * math.log(1.5) + 0.25 * math.log(0.5))) < 1e-14      # first argument weights
    assert abs(O.kl_divergence(b, a) - (0.5 * math.log(2 / 3) + 0.5 * math.log(2.0))) < 1e-14
    assert O.kl_divergence(a + 7.5, b - 3.0) == pytest.approx(O.kl_divergence(a, b), abs=1e-13)  # logits, not log-probs
    rng = np.random.default_rng(3)
    from scipy.special import rel_entr, softmax
    for _ in range(5):
        za, zb = rng.normal(size=33) * 3, rng.normal(size=33) * 3
        assert O.kl_divergence(za, za) == 0.0
        assert O.kl_divergence(za, zb) == pytest.approx(float(np.sum(rel_entr(softmax(za), softmax(zb)))), abs=1e-12)
        assert O.kl_divergence(za, zb) > 0


@pytest.mark.parametrize("layers", [(1, 1, 1), (0, 1, 2)])
def test_training_forward_rows_are_single_row_passes_over_the_stored_keys(layers):
    """The doubled sequence with its mask, written out row by row: the pseudo state of position j, step i, is one row
    at position j + i over the keys and values the causal pass stored for positions 0 .. j+i-1 (Sec. 3.3)."""
    wl = small_workload(k=3, n_layers=3, transfer_layers=layers)
    model = oracle_model(wl)
    c = model.cfg
    n = 9
    toks = [int(t) for t in counter_tokens(wl.seed, 1, n, wl.vocab)]
    z_causal, hidden, ks, vs = model.causal_forward(toks)
    for i in (1, 2, 3):
        res = O.training_forward(model, toks, i)
        assert np.max(np.abs(res["Z"] - z_causal)) < 1e-9             # hidden states never see a pseudo state
        t = layers[i - 1]
        for j in range(n):
            x = (model.w.w_transfer[i - 1] @ hidden[t][j])[None, :]
            seen = min(j + i, n)
            for layer in range(t, c.n_layers):
                x, _, _ = model.block(layer, x, np.array([j + i]), ks[layer][:seen], vs[layer][:seen],
                                      np.ones((1, seen), dtype=bool), np.ones((1, 1), dtype=bool))
            assert np.max(np.abs(model.logits(x)[0] - res["Zp"][j])) < 1e-9, (i, j)
        assert len(res["kl"]) == n - i - 1                             # the paper's index range q = 1 .. n-i-1
        want = [O.kl_divergence(res["Zp"][j], z_causal[j + i]) for j in range(n - i - 1)]
        assert np.allclose(res["kl"], want, atol=1e-14) and res["loss"] == pytest.approx(sum(want), abs=1e-13)
        assert np.all(res["kl"] > 0)


def test_training_forward_of_step_one_is_the_draft_of_inference():
    """For the first transfer step the training mask and position are those of inference (Sec. 3.3 sets the position
    id so that the two stages agree): the pseudo state of position j gives the draft distribution the decoder
    computes after a prompt of j + 1 tokens."""
    wl = small_workload(k=2, transfer_layers=(1, 1), max_cache=32)
    model = oracle_model(wl)
    toks = [int(t) for t in counter_tokens(wl.seed, 1, 8, wl.vocab)]
    res = O.training_forward(model, toks, 1)
    for j in (0, 3, 7):
        dec = O.HiddenTransferOracle(model, [-1], [0], wl.max_cache)
        dec.prefill(toks[:j + 1])
        d = dec.draft(dec.transfer())
        assert np.max(np.abs(d[0] - res["Zp"][j])) < 1e-9


@pytest.mark.parametrize("layers", [(1, 1, 1), (0, 1, 2)])
def test_training_forward_fed_true_hidden_states_reproduces_the_causal_logits(layers):
    """Mask and position id of the pseudo states, pinned without typing them again: with a map that sends every
    hidden state h_j to the true hidden state of position j + i (solved for, the h_j being linearly independent),
    pseudo state j is the real state of position j + i at position id j + i seeing positions 0 .. j+i-1 and itself,
    i.e. the causal pass, so its logits must be those of position j + i and every loss term must vanish (Sec. 3.3).
    The same map used for another step (wrong offset between position and content) must not do that."""
    wl = small_workload(k=3, n_layers=3, transfer_layers=layers, d_model=16)
    model = oracle_model(wl, make_weights(wl, wl.seed, sigma=0.4))
    n = 9
    toks = [int(t) for t in counter_tokens(wl.seed, 1, n, wl.vocab)]
    z_causal, hidden, _, _ = model.causal_forward(toks)
    for i in (1, 2, 3):
        h = hidden[layers[i - 1]]
        src, dst = h[:n - i], h[i:]                                  # W src_j = dst_j for j = 0 .. n-i-1
        assert np.linalg.matrix_rank(src) == n - i
        w_true = np.linalg.lstsq(src, dst, rcond=None)[0].T
        assert np.max(np.abs(src @ w_true.T - dst)) < 1e-9
        kept = model.w.w_transfer[i - 1]
        model.w.w_transfer[i - 1] = w_true
        res = O.training_forward(model, toks, i)
        assert np.max(np.abs(res["Zp"][:n - i] - z_causal[i:])) < 1e-7, i
        assert np.max(np.abs(res["kl"])) < 1e-12
        other = i % 3 + 1                                            # the map of step i under the position ids of another step
        if layers[other - 1] == layers[i - 1]:
            kept_other = model.w.w_transfer[other - 1]
            model.w.w_transfer[other - 1] = w_true
            off = O.training_forward(model, toks, other)
            m = n - max(i, other)
            assert np.max(np.abs(off["Zp"][:m] - z_causal[i:i + m])) > 1e-4
            model.w.w_transfer[other - 1] = kept_other
        model.w.w_transfer[i - 1] = kept
