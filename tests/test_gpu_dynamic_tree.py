"""The tree chosen at every step from the draft distributions (`ht_set_dynamic_tree`), HIP path against the oracle,
through the C ABI.  Needs a real MI355X.

The two kernels on their own: candidate log-probabilities against the fp64 log-softmax (<= 2e-5 absolute: float32
sums over the vocabulary), the tree choice bit for bit against `oracle.dynamic_tree` on the same float32 table
(ties, -inf, NaN and the largest sizes included; where the complete candidate tree is too large to enumerate, against
properties that fix the result).  Then whole decode steps: every float stage against the oracle, every integer stage
against the oracle's rule on the GPU's own numbers, the emitted text against plain greedy decoding.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from ht_inputs import WORKLOADS, make_weights, prune_tree
from oracle import ht_oracle as O
from helpers import oracle_model, prompt_of, tree_of

DEV = "cuda:0"
TOPK, WORDS = 64, 4                  # mask words per row: HT_MAX_ROWS / 64


def _B():
    import paper_2404_12022_amd.binding as B
    return B


def _H():
    import gpu_harness as H
    return H


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("rows,V,b", [(3, 32000, 10), (1, 1001, 1), (8, 40, 7), (5, 4099, 64), (2, 64, 64), (128, 515, 3)])
def test_candidate_logprobs_match_log_softmax(rows, V, b):
    B = _B()
    say(f"log-probabilities rows={rows} V={V} b={b}")
    gen = torch.Generator().manual_seed(rows * 7919 + V)
    d = (torch.randn(rows, V, generator=gen) * 3.0).float()
    d[0, : min(V, 5)] = 11.5                                     # a few equal values at the top of the first row
    dn = d.numpy().astype(np.float64)
    want = [O.candidate_logprobs(dn[i], b) for i in range(rows)]
    cand = torch.zeros(rows, TOPK, dtype=torch.int32)
    for i in range(rows):
        cand[i, :b] = torch.tensor(want[i][0], dtype=torch.int32)
    lp = torch.full((rows, TOPK), 7.0, dtype=torch.float32, device=DEV)
    B.ht_candidate_logprobs(d.to(DEV), cand.to(DEV), b, lp)
    torch.cuda.synchronize()
    got = lp.cpu().numpy()
    err = float(np.max(np.abs(got[:, :b].astype(np.float64) - np.stack([w[1] for w in want]))))
    say(f"  max-abs error {err:.2e}")
    assert err <= 2e-5
    assert np.all(got[:, b:] == 7.0)                             # nothing past the b entries is written
    assert np.all(got[:, :b] <= 0)


def _run_tree_kernel(lp_table, cand_table, root, k, b, T):
    """lp_table, cand_table: numpy [k, b].  Returns (parent, depth, rank, anc [T, 2] uint64, tokens)."""
    B = _B()
    lp = torch.zeros(k, TOPK, dtype=torch.float32)
    cand = torch.zeros(k, TOPK, dtype=torch.int32)
    lp[:, :b] = torch.from_numpy(np.ascontiguousarray(lp_table, dtype=np.float32))
    cand[:, :b] = torch.from_numpy(np.ascontiguousarray(cand_table, dtype=np.int32))
    out = [torch.full((T,), -7, dtype=torch.int32, device=DEV) for _ in range(4)]
    anc = torch.zeros(T, WORDS, dtype=torch.int64, device=DEV)
    B.ht_dynamic_tree(lp.to(DEV), cand.to(DEV), torch.tensor([root], dtype=torch.int32, device=DEV), k, b, T,
                      out[0], out[1], out[2], anc, out[3])
    torch.cuda.synchronize()
    parent, depth, rank, tokens = ([int(x) for x in t.cpu()] for t in out)
    return parent, depth, rank, anc.cpu().numpy().view(np.uint64), tokens


def _check_tables(parent, depth, rank, anc, tokens, cand_table, root):
    T = len(parent)
    assert depth == O.tree_depth(parent)
    want_anc = O.ancestor_matrix(parent)
    for v in range(T):
        bits = [bool((int(anc[v, u >> 6]) >> (u & 63)) & 1) for u in range(64 * WORDS)]
        assert bits[:T] == [bool(x) for x in want_anc[v]] and not any(bits[T:]), f"ancestor mask of node {v}"
    assert tokens == [root] + [int(cand_table[depth[v] - 1][rank[v]]) for v in range(1, T)]


def _tables(kind, k, b, rng):
    """Candidate log-probability rows, best first."""
    if kind == "softmax":                                        # what a draft gives: top b of a log-softmax
        return np.stack([O.candidate_logprobs(rng.normal(size=4 * b + 3) * 2.5, b)[1] for _ in range(k)]).astype(np.float32)
    if kind == "ties":                                           # few distinct values: the tie rules decide most picks
        return -np.sort(rng.integers(0, 3, size=(k, b)), axis=1).astype(np.float32) * 0.25
    if kind == "uniform":
        return np.full((k, b), -np.log(b), dtype=np.float32)
    if kind == "holes":                                          # impossible candidates and NaN at the ends of the rows
        t = -np.sort(rng.random(size=(k, b)), axis=1).astype(np.float32)
        t[:, b - b // 3:] = -np.inf
        if b > 2:
            t[k - 1, b - 1] = np.nan
        return t
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["softmax", "ties", "uniform", "holes"])
def test_tree_choice_is_the_oracle_rule_bit_for_bit(kind):
    rng = np.random.default_rng({"softmax": 1, "ties": 2, "uniform": 3, "holes": 4}[kind])
    shapes = [(1, 1), (1, 64), (2, 2), (2, 3), (2, 11), (3, 2), (3, 4), (3, 10), (4, 3), (4, 6), (5, 3), (6, 2), (8, 2), (8, 3)]
    cases = 0
    for k, b in shapes:
        room = sum(b ** e for e in range(1, k + 1))
        if room > 12000:
            continue
        sizes = sorted({1, 2, min(room + 1, 128), min(room + 1, 65), 1 + room // 2 if room // 2 < 128 else 100})
        lp = _tables(kind, k, b, rng)
        cand = rng.integers(0, 32000, size=(k, b))
        for T in sizes:
            say(f"tree choice {kind} k={k} b={b} T={T}")
            parent, depth, rank, anc, tokens = _run_tree_kernel(lp, cand, 4242, k, b, T)
            assert (parent, rank) == O.dynamic_tree(lp, T), (kind, k, b, T)
            _check_tables(parent, depth, rank, anc, tokens, cand, 4242)
            cases += 1
    say(f"{kind}: {cases} trees equal the oracle's")


def test_tree_choice_at_the_largest_sizes():
    """k = 8 levels of 64 candidates, 128 nodes: the complete tree (64^8 nodes) cannot be enumerated, so the result
    is checked by what fixes it: a valid parent-closed tree whose nodes come in non-ascending (score, then the tie
    rules) order, whose every left-out next sibling and first child comes after the last node taken."""
    rng = np.random.default_rng(77)
    k, b, T = 8, 64, 128
    for kind in ("softmax", "ties"):
        lp = _tables(kind, k, b, rng)
        cand = rng.integers(0, 32000, size=(k, b))
        say(f"largest tree choice, {kind}")
        parent, depth, rank, anc, tokens = _run_tree_kernel(lp, cand, 9, k, b, T)
        _check_tables(parent, depth, rank, anc, tokens, cand, 9)
        assert parent[0] == -1 and all(0 <= parent[v] < v for v in range(1, T)) and max(depth) <= k
        paths, score = [()], [np.float32(0)]
        for v in range(1, T):
            paths.append(paths[parent[v]] + (rank[v],))
            score.append(np.float32(score[parent[v]] + lp[depth[v] - 1, rank[v]]))
        assert len(set(paths)) == T
        key = lambda v: (-float(score[v]), depth[v], paths[v])
        assert all(key(v) < key(v + 1) for v in range(1, T - 1))
        taken = set(paths)
        for v in range(T):                                      # the frontier the walk left behind
            nxt = []
            if v and rank[v] + 1 < b:
                nxt.append((paths[v][:-1] + (rank[v] + 1,), score[parent[v]], depth[v]))
            if depth[v] < k:
                nxt.append((paths[v] + (0,), score[v], depth[v] + 1))
            for path, base, dep in nxt:
                if path not in taken:
                    s = np.float32(base + lp[dep - 1, path[-1]])
                    assert (-float(s), dep, path) > key(T - 1), f"node {path} should have been taken"


@pytest.mark.parametrize("name,T,b", [("tiny", 8, 3), ("tiny_k3", 16, 4), ("tiny_t123", 12, 3), ("tiny", 1, 1), ("tiny", 7, 2)])
def test_tiny_fp32_steps_with_a_tree_chosen_every_step(name, T, b):
    H = _H()
    wl = WORKLOADS[name]
    say(f"dynamic tree end-to-end {name} T={T} b={b}")
    sc = H.StepCompare(wl, dynamic=(T, b))
    sc.check_prefill()
    out, shapes = [], set()
    for step in range(12):
        r = sc.step_dynamic()
        out += r["emitted"]
        shapes.add(tuple(r["parent"]))
    assert out == sc.model.ar_greedy(sc.prompt, len(out))            # losslessness on the GPU
    sc.check_cache("after 12 steps")
    say(f"{name}: {len(shapes)} different trees in 12 steps, {len(out)} tokens, largest logit error {sc.max_err:.3e}")
    if T > 2 and b > 1:
        assert len(shapes) > 1
    sc.gpu.close()


@pytest.mark.parametrize("name", ["tiny_bf16", "tiny_t123_bf16"])
def test_tiny_bf16_steps_with_a_tree_chosen_every_step(name):
    H = _H()
    wl = WORKLOADS[name]
    say(f"dynamic tree end-to-end {name}")
    sc = H.StepCompare(wl, dynamic=(8, 3))
    sc.check_prefill()
    same = 0
    for step in range(12):
        r = sc.step_dynamic(exact=False)
        same += (r["parent"], r["rank"]) == r["own_tree"]
    sc.check_cache("after 12 steps")
    say(f"{name}: {same} of 12 trees equal the fp64 oracle's own, worst logit error / bound {sc.max_err:.3f}")
    sc.gpu.close()


def test_device_resident_loop_with_a_tree_chosen_every_step():
    """`ht_decode_steps` in this mode against single steps of the same library (same kernels, same values), and both
    against plain greedy decoding."""
    B, H = _B(), _H()
    wl = WORKLOADS["tiny_k3"].with_(max_cache=256)
    a, b = H.gpu_model(wl, max_tree=16), H.gpu_model(wl, max_tree=16)
    prompt = prompt_of(wl)
    for g in (a, b):
        g.ht_set_dynamic_tree(16, 4)
        g.ht_prefill(prompt)
    say("device-resident loop with a dynamic tree")
    counts, toks, root = a.ht_decode_steps(20)
    ref_counts, ref_toks = [], []
    for _ in range(20):
        b.ht_transfer(None, None)
        b.ht_tree_verify_step(None, None, None)
        m, emitted, ref_root, _ = b.ht_accept_and_compact()
        ref_counts.append(m)
        ref_toks += emitted
    assert (counts, toks, root) == (ref_counts, ref_toks, ref_root)
    want = oracle_model(wl).ar_greedy(prompt, len(toks) + 1)
    assert toks == want[:-1] and root == want[-1]
    assert torch.equal(a.ht_get_buffer(B.HT_BUF_TREE_PARENT), b.ht_get_buffer(B.HT_BUF_TREE_PARENT))
    a.close()
    b.close()


def test_switching_between_fixed_and_chosen_trees_and_error_codes():
    B, H = _B(), _H()
    wl = WORKLOADS["tiny"].with_(max_cache=256)
    parent, rank = tree_of(wl)
    gpu = H.gpu_model(wl, max_tree=16)
    prompt = prompt_of(wl)
    gpu.ht_prefill(prompt)
    for T, b in ((17, 4), (0, 2), (8, 0), (8, 65), (8, 2)):          # max_tree 16; 2 + 4 = 6 nodes below the root at most
        with pytest.raises(B.HTError) as e:
            gpu.ht_set_dynamic_tree(T, b)
        assert e.value.code == B.HT_ETREE, (T, b)
    out = []
    gpu.ht_set_dynamic_tree(7, 2)                                    # the complete tree: every step the same shape
    for step in range(3):
        gpu.ht_transfer(None, None)
        gpu.ht_tree_verify_step(None, None, None)
        out += gpu.ht_accept_and_compact()[1]
        shape = O.tree_depth(gpu.ht_get_buffer(B.HT_BUF_TREE_PARENT).tolist())
        assert sorted(shape) == [0, 1, 1, 2, 2, 2, 2]
    with pytest.raises(B.HTError) as e:
        gpu.ht_set_fused_nodes([0])
    assert e.value.code == B.HT_ESTATE
    before = gpu.ht_get_buffer(B.HT_BUF_TREE_PARENT).tolist()
    gpu.ht_set_fused_nodes([])                                       # switching it off is always allowed and changes nothing
    assert gpu.ht_get_buffer(B.HT_BUF_TREE_PARENT).tolist() == before
    gpu.ht_transfer(None, None)
    with pytest.raises(B.HTError) as e:
        gpu.ht_tree_verify_step(torch.zeros(7, dtype=torch.int32, device=DEV), None, None)
    assert e.value.code == B.HT_ESTATE
    gpu.ht_set_tree(parent, rank)                                    # back to the fixed tree
    for step in range(3):
        gpu.ht_transfer(None, None)
        gpu.ht_tree_verify_step(None, None, None)
        out += gpu.ht_accept_and_compact()[1]
    assert gpu.ht_get_buffer(B.HT_BUF_TREE_PARENT).tolist() == list(parent)
    gpu.ht_set_dynamic_tree(12, 3)
    for step in range(3):
        gpu.ht_transfer(None, None)
        gpu.ht_tree_verify_step(None, None, None)
        out += gpu.ht_accept_and_compact()[1]
    assert out == oracle_model(wl).ar_greedy(prompt, len(out))
    gpu.close()


def test_llama7b_width_two_layers_with_a_tree_chosen_every_step():
    """Full 7B widths and vocabulary, 64 nodes among the 10 best candidates of 3 positions (1110 possible nodes),
    depth cut to 2 layers so the fp64 oracle finishes in seconds."""
    H = _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), prompt_len=200, max_cache=512)
    say("7B-width 2 layers, dynamic tree: generating weights")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    sc = H.StepCompare(wl, tensors_gpu=tensors, tensors_cpu=cpu_tensors, dynamic=(64, 10))
    sc.check_prefill()
    for step in range(2):
        r = sc.step_dynamic(exact=False)
        say(f"  step {step}: depth profile {np.bincount(O.tree_depth(r['parent'])).tolist()}, accepted {r['m']}, "
            f"tree equals the fp64 oracle's own: {(r['parent'], r['rank']) == r['own_tree']}")
    sc.gpu.close()


@pytest.mark.parametrize("seed", [f"any{i}" for i in range(6)] + [f"packed{i}" for i in range(6)])
def test_random_model_shapes_with_a_tree_chosen_every_step(seed):
    """The random shapes of the fixed-tree suite (grouped heads, odd widths, 1..5 transfer steps at different layers,
    both kernel families), decoding with a tree of the same size chosen at every step."""
    from test_gpu_parity import _random_shape, _random_packed_shape
    H = _H()
    wl, _, _ = _random_shape(int(seed[3:])) if seed.startswith("any") else _random_packed_shape(int(seed[6:]))
    b = 2
    while sum(b ** e for e in range(1, wl.k + 1)) < wl.tree_size - 1:
        b += 1
    b = min(b + 1, 64, wl.vocab)
    wl = wl.with_(max_cache=wl.max_cache + 64)
    say(f"dynamic tree, random shape {seed}: {wl.dtype} layers={wl.n_layers} d={wl.d_model} heads={wl.n_heads}/{wl.n_kv_heads}x"
        f"{wl.head_dim} vocab={wl.vocab} k={wl.k} t={wl.transfer_layers} T={wl.tree_size} b={b} prompt {wl.prompt_len}")
    sc = H.StepCompare(wl, dynamic=(wl.tree_size, b))
    sc.check_prefill()
    for step in range(4):
        sc.step_dynamic(exact=False)
    sc.check_cache("after 4 steps")
    sc.gpu.close()


def test_drafting_step_with_a_chosen_tree_replayed_from_a_graph():
    """Transfer, draft pass, top-k, log-probabilities, tree choice and verify pass captured in one HIP graph: every
    replay, with eager work of the same model in between, gives the tree, tokens and logits of the eager call."""
    B, H = _B(), _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), prompt_len=90, max_cache=256)
    T, b = 32, 6
    model = H.gpu_model(wl, make_weights(wl, wl.seed, H.DEV, torch.bfloat16), max_tree=T)
    model.ht_set_dynamic_tree(T, b)
    model.ht_prefill(prompt_of(wl))
    z_e = torch.empty(T, wl.vocab, dtype=torch.float32, device=DEV)
    g_e = torch.empty(T, dtype=torch.int32, device=DEV)
    z_g, g_g = torch.empty_like(z_e), torch.empty_like(g_e)

    def eager():
        model.ht_transfer(None, None)
        model.ht_tree_verify_step(None, g_e, z_e)
        torch.cuda.synchronize()
        return (model.ht_get_buffer(B.HT_BUF_TREE_PARENT).clone(), model.ht_get_buffer(B.HT_BUF_TREE_RANK).clone(),
                model.ht_get_buffer(B.HT_BUF_TREE_TOKENS).clone())

    want = eager()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        model.ht_transfer(None, None)
        model.ht_tree_verify_step(None, g_g, z_g)
    say("graph replay of a drafting step with a chosen tree")
    for replay in range(4):
        z_g.zero_()
        g_g.zero_()
        other = torch.full((T,), 5 + replay, dtype=torch.int32, device=DEV)
        model.ht_set_tree(*prune_tree(wl.branching, T))          # eager work between the replays rewrites the tables
        model.ht_tree_verify_step(other, g_e, z_e)
        model.ht_set_dynamic_tree(T, b)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (model.ht_get_buffer(B.HT_BUF_TREE_PARENT).clone(), model.ht_get_buffer(B.HT_BUF_TREE_RANK).clone(),
               model.ht_get_buffer(B.HT_BUF_TREE_TOKENS).clone())
        assert all(torch.equal(a, c) for a, c in zip(got, want)), f"replay {replay}: tree or tokens differ"
        again = eager()
        assert all(torch.equal(a, c) for a, c in zip(again, want))
        assert torch.equal(g_g, g_e), f"replay {replay}: arg-max differs from the eager pass"
        assert torch.equal(z_g, z_e), f"replay {replay}: logits differ from the eager pass"
    del graph
    model.close()
