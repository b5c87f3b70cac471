"""CPU oracle for Hidden Transfer tree-verify decoding.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy implementation of what the GPU library computes, written from the
paper (arXiv 2404.12022) and used only by the tests, the smoke check and the benchmark's CPU
baseline.  It shares no code with the HIP path and must never be imported by the product.

What is written out here, and the passage each part follows:

  * Llama-style decoder block with arbitrary visibility mask and position ids
    (Sec. 3.1 problem formulation; Sec. 4.1 names LLaMA-2 / Vicuna as the architecture).
  * Plain greedy autoregressive decoding by full causal recompute: the definition of a
    correct output (Sec. 3.1; Sec. 4.1 "identical to standard auto-regressive decoding").
  * Hidden transfer  p_i = W^i_{t_i} h^{t_i}  (Sec. 3.2; equation of Sec. 3.3).
  * Pseudo rows continue through blocks t_i+1..L, seeing the context, earlier pseudo rows and
    themselves, at position (source position + i), decoded with the original LM head
    (Sec. 1, Sec. 3.2, Sec. 3.3 position-id sentence, Sec. 4.4 "No masked" setting).
  * Candidate tree, flattening, ancestor-only mask, original positional indices
    (Sec. 3.4 and 3.4.1).
  * Greedy verification: last accepted position, next token (Fig. 2 caption; Sec. 3.4).
  * Both inference schedules: "draft after accept" (S1) and the paper's fused
    "verify and draft in the same forward" (S2, Fig. 2 caption / Sec. 3.4 last sentence).
  * The forward pass of the training stage and its distillation loss for one transfer step
    (Sec. 3.3: the doubled sequence of hidden and pseudo hidden states, its attention mask and
    position ids, the KL term per position): `training_forward`.  Forward only; the paper trains
    the maps with this loss, which needs its dataset and is outside this build.
  * A tree chosen anew at every step from the draft distributions (`candidate_logprobs`,
    `dynamic_tree`).  The paper decodes with a pre-defined tree (Sec. 3.4.1) and names the choice of
    the tree's structure as what the speed depends on and as future work (Limitation section); the
    rule here is this build's own, defined by these two functions: the nodes a greedy verification
    is most likely to reach if the draft distributions were the model's.

Arithmetic: weights exactly as stored (fp32 or bf16 widened to fp64), every accumulation in
fp64, no intermediate rounding.  Index conventions: positions are 0-based, the cache holds
positions 0..n-1, the tree root sits at position n, a node of depth e at n+e, and pseudo row
i (1-based) made from the token at position s sits at s+i.  "Layer t" means the residual
stream after t complete blocks (t = 0 is the embedding output).

Pins: every function here is pinned by tests/test_oracle_*.py (closed forms, loop-level brute
force, the causal-path invariant, losslessness against `ar_greedy`, exhaustive acceptance
search, S1 == S2; the dynamic tree against an exhaustive search over all trees of its size; the
training forward row by row against single-row passes over stored keys, for step 1 against
the inference-time draft, and for every step against the causal logits when the map sends each hidden
state to the true hidden state of the position it stands for).
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# ------------------------------------------------------------------------------------ model
@dataclass
class OracleConfig:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    k: int
    transfer_layers: Tuple[int, ...]
    rms_eps: float = 1e-5
    rope_base: float = 10000.0


class OracleWeights:
    """fp64 copies of the stored weights.  Matrices are [out, in]; y = x @ W.T."""

    def __init__(self, tensors: Dict[str, object]):
        def cv(a):
            if a is None:
                return None
            if hasattr(a, "detach"):                      # torch tensor (any dtype, any device)
                a = a.detach().to("cpu").double().numpy()
            return np.asarray(a, dtype=np.float64)

        self.tok_emb = cv(tensors["tok_emb"])
        self.final_norm = cv(tensors["final_norm"])
        self.lm_head = cv(tensors["lm_head"])
        self.w_transfer = [cv(a) for a in tensors["w_transfer"]]
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            setattr(self, name, [cv(a) for a in tensors[name]])


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y = x W^T for a row-major [out, in] matrix: the textbook matrix product, in fp64."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain, row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding on x[R, H, hd] at integer positions pos[R].

    Pair (j, j + hd/2) is rotated by the angle pos * base^(-2j/hd), j = 0..hd/2-1.
    """
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]        # [R, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def masked_attention(q: np.ndarray, keys: np.ndarray, values: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """softmax over the visible keys of q.k / sqrt(hd), times values.

    q[R, Hq, hd]; keys, values[S, Hkv, hd]; visible[R, S] bool.  Query head h reads key/value
    head h // (Hq / Hkv).  Returns [R, Hq, hd].
    """
    r, hq, hd = q.shape
    hkv = keys.shape[1]
    group = hq // hkv
    out = np.zeros_like(q)
    for h in range(hq):
        kh, vh = keys[:, h // group, :], values[:, h // group, :]
        score = q[:, h, :] @ kh.T / np.sqrt(hd)                               # [R, S]
        score = np.where(visible, score, -np.inf)
        score = score - score.max(axis=1, keepdims=True)
        p = np.exp(score)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


class OracleModel:
    def __init__(self, cfg: OracleConfig, weights: OracleWeights):
        self.cfg, self.w = cfg, weights

    def embed(self, tokens: Sequence[int]) -> np.ndarray:
        return self.w.tok_emb[np.asarray(tokens, dtype=np.int64)].copy()

    def block(self, layer: int, x: np.ndarray, pos: np.ndarray,
              k_old: np.ndarray, v_old: np.ndarray, vis_old: np.ndarray, vis_new: np.ndarray):
        """One decoder block (0-based `layer`) on rows x[R, d].

        The rows attend to already-stored keys k_old/v_old[S, Hkv, hd] where vis_old[R, S] and to
        each other's fresh keys where vis_new[R, R].  Returns (x_out, k_new, v_new); k_new is
        post-rotary, as stored in a cache.
        """
        c, w = self.cfg, self.w
        r = x.shape[0]
        u = rms_norm(x, w.attn_norm[layer], c.rms_eps)
        q = linear(u, w.wq[layer]).reshape(r, c.n_heads, c.head_dim)
        k = linear(u, w.wk[layer]).reshape(r, c.n_kv_heads, c.head_dim)
        v = linear(u, w.wv[layer]).reshape(r, c.n_kv_heads, c.head_dim)
        q, k = rope(q, pos, c.rope_base), rope(k, pos, c.rope_base)
        keys = np.concatenate([k_old, k], axis=0)
        vals = np.concatenate([v_old, v], axis=0)
        vis = np.concatenate([vis_old, vis_new], axis=1)
        a = masked_attention(q, keys, vals, vis).reshape(r, c.n_heads * c.head_dim)
        x = x + linear(a, w.wo[layer])
        u2 = rms_norm(x, w.ffn_norm[layer], c.rms_eps)
        x = x + linear(silu(linear(u2, w.w_gate[layer])) * linear(u2, w.w_up[layer]), w.w_down[layer])
        return x, k, v

    def logits(self, x: np.ndarray) -> np.ndarray:
        return linear(rms_norm(x, self.w.final_norm, self.cfg.rms_eps), self.w.lm_head)

    # ---- plain causal forward, full recompute: the textbook definition everything is pinned to
    def causal_forward(self, tokens: Sequence[int]):
        """Returns (logits[n, V], hidden[L+1][n, d], K[L][n, Hkv, hd], V[L][...])."""
        c = self.cfg
        n = len(tokens)
        x = self.embed(tokens)
        pos = np.arange(n)
        tri = np.tril(np.ones((n, n), dtype=bool))
        empty = np.zeros((0, c.n_kv_heads, c.head_dim))
        none_vis = np.zeros((n, 0), dtype=bool)
        hidden, ks, vs = [x], [], []
        for layer in range(c.n_layers):
            x, k, v = self.block(layer, x, pos, empty, empty, none_vis, tri)
            hidden.append(x)
            ks.append(k)
            vs.append(v)
        return self.logits(x), hidden, ks, vs

    def ar_greedy(self, prompt: Sequence[int], steps: int) -> List[int]:
        """x_{j+1} = argmax LM(x_0..x_j), lowest id on ties; one token at a time, no cache."""
        seq = list(prompt)
        for _ in range(steps):
            z, _, _, _ = self.causal_forward(seq)
            seq.append(int(np.argmax(z[-1])))
        return seq[len(prompt):]


# ------------------------------------------------------------------------------------ training stage (Sec. 3.3)
def kl_divergence(za: np.ndarray, zb: np.ndarray) -> float:
    """KL(A || B) = sum_v A_v (log A_v - log B_v) of the softmax distributions of two logit rows."""
    la = za - np.max(za)
    la = la - np.log(np.sum(np.exp(la)))
    lb = zb - np.max(zb)
    lb = lb - np.log(np.sum(np.exp(lb)))
    return float(np.sum(np.exp(la) * (la - lb)))


def training_forward(model: OracleModel, tokens: Sequence[int], step: int):
    """Forward pass of the training stage for transfer step `step` (1-based i of Sec. 3.3) over n tokens.

    The tokens run causally up to the transfer layer t_i; every hidden state h_j becomes a pseudo state
    W_i h_j; the 2n rows (hidden states, then pseudo states) go on through blocks t_i+1..L.  Hidden states
    attend causally among themselves.  Pseudo state j (0-based; it stands for position j + i) has position
    id j + i and attends to the hidden states of positions 0 .. j+i-1 and to itself, to no other pseudo
    state.  All rows pass the original LM head.  The loss adds KL(P~_j || P_{j+i}), the pseudo state's
    distribution against that of the hidden state it stands for, with the first argument weighting the
    log ratio, over the paper's index range q = 1 .. n-i-1 (1-based), i.e. j = 0 .. n-i-2.
    Returns dict(Z[n, V] logits of the hidden states, Zp[n, V] logits of the pseudo states, kl[n-i-1], loss)."""
    c = model.cfg
    n, i = len(tokens), step
    t = c.transfer_layers[i - 1]
    _, hidden, _, _ = model.causal_forward(tokens)
    h = hidden[t]
    x = np.concatenate([h, linear(h, model.w.w_transfer[i - 1])], axis=0)
    pos = np.concatenate([np.arange(n), np.arange(n) + i])
    vis = np.zeros((2 * n, 2 * n), dtype=bool)
    for a in range(n):
        vis[a, :a + 1] = True                               # hidden state a: positions 0 .. a
        vis[n + a, :min(a + i, n)] = True                   # pseudo state a: hidden states 0 .. a+i-1
        vis[n + a, n + a] = True                            # and itself
    empty = np.zeros((0, c.n_kv_heads, c.head_dim))
    none_vis = np.zeros((2 * n, 0), dtype=bool)
    for layer in range(t, c.n_layers):
        x, _, _ = model.block(layer, x, pos, empty, empty, none_vis, vis)
    z_all = model.logits(x)
    z, zp = z_all[:n], z_all[n:]
    kl = np.array([kl_divergence(zp[j], z[j + i]) for j in range(max(n - i - 1, 0))])
    return dict(Z=z, Zp=zp, kl=kl, loss=float(np.sum(kl)))


# ------------------------------------------------------------------------------------ tree helpers
def tree_depth(parent: Sequence[int]) -> List[int]:
    depth = [0] * len(parent)
    for v in range(1, len(parent)):
        depth[v] = depth[parent[v]] + 1
    return depth


def ancestor_matrix(parent: Sequence[int]) -> np.ndarray:
    """anc[v, u] = True iff u is v or an ancestor of v (a token attends only to these, Sec. 3.4.1)."""
    t = len(parent)
    anc = np.zeros((t, t), dtype=bool)
    for v in range(t):
        if parent[v] >= 0:
            anc[v] = anc[parent[v]]
        anc[v, v] = True
    return anc


def top_candidates(row: np.ndarray, b: int) -> List[int]:
    """The b largest entries of a logit row, ordered by (value descending, id ascending)."""
    order = np.lexsort((np.arange(row.shape[0]), -row))
    return [int(j) for j in order[:b]]


def candidate_logprobs(row: np.ndarray, b: int) -> Tuple[List[int], np.ndarray]:
    """The b best tokens of one draft distribution (value descending, id ascending) and their log-softmax
    values  z_j - log(sum_v exp z_v)  over the whole vocabulary."""
    z = np.asarray(row, dtype=np.float64)
    ids = top_candidates(z, b)
    peak = np.max(z)
    lse = peak + np.log(np.sum(np.exp(z - peak)))
    return ids, np.array([z[j] - lse for j in ids])


def dynamic_tree(lp: np.ndarray, T: int) -> Tuple[List[int], List[int]]:
    """Tree of T nodes (root included) for one step, from lp[e - 1, r] = log-probability of the r-th best
    candidate of pseudo position e (rows sorted best first, all values <= 0).

    The drafts of the k positions do not depend on one another (Sec. 3.2: every pseudo state is made from the
    same hidden state), so a node whose path from the root picks ranks (r_1, .., r_e) is reached by a greedy
    verification with probability exp(score), score = lp[0, r_1] + .. + lp[e-1, r_e], if the drafts were
    exact.  The tree is the T - 1 nodes of the complete b-ary tree of depth k that come first in the order
    (score descending, depth ascending, rank path ascending); a child never scores above its parent, so the
    set is closed under taking parents and maximises the expected number of accepted candidates.  Nodes are
    numbered in that order after the root.  The score is accumulated from the root down in lp's own dtype
    (the decision is taken in the precision of the caller's numbers); NaN counts as -inf.
    Returns (parent, rank) as `ht_set_tree` takes them."""
    lp = np.asarray(lp)
    k, b = lp.shape
    kind = lp.dtype.type
    nodes = []
    for e in range(1, k + 1):
        for path in itertools.product(range(b), repeat=e):
            score = kind(0)
            for level, r in enumerate(path):
                term = lp[level, r]
                score = score + (term if term == term else kind(-np.inf))
            nodes.append((-float(score), e, path))
    if T < 1 or T - 1 > len(nodes):
        raise ValueError(f"a tree of {T} nodes does not fit {k} levels of {b} candidates")
    nodes.sort()
    chosen = [path for _, _, path in nodes[:T - 1]]
    index = {(): 0}
    for v, path in enumerate(chosen, start=1):
        index[path] = v
    parent, rank = [-1], [0]
    for path in chosen:
        parent.append(index[path[:-1]])          # KeyError would mean the set is not closed under parents
        rank.append(path[-1])
    return parent, rank


def accept_walk(parent: Sequence[int], tok: Sequence[int], g: Sequence[int]) -> Tuple[List[int], int]:
    """Greedy verification: follow, from the root, the first child (lowest index) whose token
    equals the model's greedy choice after its parent; stop when no child matches.
    Returns (path of node ids, next root token)."""
    t = len(parent)
    path, cur = [0], 0
    while True:
        nxt = -1
        for c in range(cur + 1, t):
            if parent[c] == cur and tok[c] == g[cur]:
                nxt = c
                break
        if nxt < 0:
            break
        path.append(nxt)
        cur = nxt
    return path, int(g[cur])


# ------------------------------------------------------------------------------------ decoder
class HiddenTransferOracle:
    """Stateful step-by-step decoder (schedule S1) plus the fused schedule S2 for cross-checking.

    State: KV cache of n tokens, pending root token (the greedy token for position n, not yet in
    the cache), and for every distinct transfer layer t the residual h^t of the last cached token.
    """

    def __init__(self, model: OracleModel, parent: Sequence[int], rank: Sequence[int], capacity: int):
        self.m, self.cfg = model, model.cfg
        c = self.cfg
        self.capacity = capacity
        self.K = [np.zeros((capacity, c.n_kv_heads, c.head_dim)) for _ in range(c.n_layers)]
        self.V = [np.zeros((capacity, c.n_kv_heads, c.head_dim)) for _ in range(c.n_layers)]
        self.n = 0
        self.root: Optional[int] = None
        self.h_src: Dict[int, np.ndarray] = {}
        self.set_tree(parent, rank)

    def set_tree(self, parent: Sequence[int], rank: Sequence[int]) -> None:
        """The tree of the following steps (a static tree is set once, a dynamic one before every verification)."""
        self.parent, self.rank = list(parent), list(rank)
        self.depth = tree_depth(parent)
        self.T = len(parent)
        self.anc = ancestor_matrix(parent)
        # candidates needed per depth: 1 + the largest rank used at that depth
        self.width = [0] * (max(self.depth) + 1)
        for v in range(1, self.T):
            self.width[self.depth[v]] = max(self.width[self.depth[v]], self.rank[v] + 1)

    # -- step 0
    def prefill(self, prompt: Sequence[int]) -> None:
        z, hidden, ks, vs = self.m.causal_forward(prompt)
        p = len(prompt)
        for layer in range(self.cfg.n_layers):
            self.K[layer][:p], self.V[layer][:p] = ks[layer], vs[layer]
        self.n = p
        self.root = int(np.argmax(z[-1]))
        self.h_src = {t: hidden[t][-1].copy() for t in set(self.cfg.transfer_layers)}

    # -- step 1
    def transfer(self) -> List[np.ndarray]:
        """p_i = W_i h^{t_i} for i = 1..k: a bare matrix product, no bias, norm or residual."""
        return [linear(self.h_src[t], self.m.w.w_transfer[i]) for i, t in enumerate(self.cfg.transfer_layers)]

    # -- step 2
    def draft(self, pseudo: List[np.ndarray]) -> np.ndarray:
        """Pseudo row i (1-based) joins before block t_i+1 at position n-1+i and sees the whole
        cache, pseudo rows j < i and itself.  Returns D[k, V]; their keys/values are discarded."""
        c = self.cfg
        n = self.n
        rows: List[int] = []
        x = np.zeros((0, c.d_model))
        for layer in range(c.n_layers):            # `layer` is 0-based: block layer+1
            for i, t in enumerate(c.transfer_layers):
                if t == layer:                      # joins after t blocks, i.e. before block t+1
                    rows.append(i)
                    x = np.concatenate([x, pseudo[i][None, :]], axis=0)
            if not rows:
                continue
            assert rows == sorted(rows)
            r = len(rows)
            pos = np.array([n + i for i in rows])   # n-1+(i+1)
            vis_old = np.ones((r, n), dtype=bool)
            vis_new = np.array([[rows[b] <= rows[a] for b in range(r)] for a in range(r)], dtype=bool)
            x, _, _ = self.m.block(layer, x, pos, self.K[layer][:n], self.V[layer][:n], vis_old, vis_new)
        assert rows == list(range(c.k))
        return self.m.logits(x)

    # -- steps 3, 4
    def candidates(self, d: np.ndarray) -> List[List[int]]:
        """cand[e] for depth e = 1..k (index 0 unused): top-width[e] tokens of D_e."""
        cand: List[List[int]] = [[]]
        for e in range(1, len(self.width)):
            cand.append(top_candidates(d[e - 1], self.width[e]))
        return cand

    def build_tree(self, cand: List[List[int]]) -> List[int]:
        tok = [int(self.root)]
        for v in range(1, self.T):
            tok.append(cand[self.depth[v]][self.rank[v]])
        return tok

    # -- step 5
    def verify(self, tok: Sequence[int]):
        """One forward of the flattened tree.  Row v sees cache[0, n) and its ancestors-or-self,
        sits at position n + depth[v]; its key/value go to slot n + v.  Returns
        (Z[T, V], g[T], H[t][T, d] for each distinct transfer layer)."""
        c, n, t_rows = self.cfg, self.n, self.T
        assert n + t_rows <= self.capacity
        x = self.m.embed(tok)
        pos = np.array([n + e for e in self.depth])
        vis_old = np.ones((t_rows, n), dtype=bool)
        saved: Dict[int, np.ndarray] = {}
        if 0 in c.transfer_layers:
            saved[0] = x.copy()
        for layer in range(c.n_layers):
            x, k, v = self.m.block(layer, x, pos, self.K[layer][:n], self.V[layer][:n], vis_old, self.anc)
            self.K[layer][n:n + t_rows], self.V[layer][n:n + t_rows] = k, v
            if layer + 1 in c.transfer_layers:
                saved[layer + 1] = x.copy()
        z = self.m.logits(x)
        return z, [int(j) for j in np.argmax(z, axis=1)], saved

    # -- steps 6, 7
    def accept_and_compact(self, tok: Sequence[int], g: Sequence[int], saved: Dict[int, np.ndarray]):
        path, new_root = accept_walk(self.parent, tok, g)
        n = self.n
        for layer in range(self.cfg.n_layers):
            for j, node in enumerate(path):         # ascending j; path[j] >= j so in place is safe
                self.K[layer][n + j] = self.K[layer][n + node]
                self.V[layer][n + j] = self.V[layer][n + node]
        emitted = [int(tok[v]) for v in path]
        self.n = n + len(path)
        self.h_src = {t: h[path[-1]].copy() for t, h in saved.items()}
        self.root = new_root
        return path, emitted

    def step(self, forced_tokens: Optional[Sequence[int]] = None, dynamic: Optional[Tuple[int, int]] = None):
        """One full S1 step.  Returns a dict of every intermediate object.
        dynamic = (T, b): the step first chooses its own tree of T nodes among the b best candidates of every
        pseudo position (`dynamic_tree` on the fp64 log-probabilities)."""
        pseudo = self.transfer()
        d = self.draft(pseudo)
        if dynamic is not None:
            size, b = dynamic
            lp = np.stack([candidate_logprobs(d[e], b)[1] for e in range(self.cfg.k)])
            self.set_tree(*dynamic_tree(lp, size))
        cand = self.candidates(d)
        tok = list(forced_tokens) if forced_tokens is not None else self.build_tree(cand)
        z, g, saved = self.verify(tok)
        path, emitted = self.accept_and_compact(tok, g, saved)
        return dict(pseudo=pseudo, D=d, cand=cand, tok=tok, Z=z, g=g, H=saved, path=path, emitted=emitted,
                    root=self.root, n=self.n)

    # -- fused schedule: verify the tree and draft for every node in the same forward
    def fused_verify_and_draft(self, tok: Sequence[int]):
        """Schedule S2.  Besides the T tree rows, every tree node v gets k pseudo rows: row (v, i)
        is W_i applied to v's own layer-t_i residual, joins before block t_i+1 at position
        pos(v) + i and sees cache, ancestors-or-self of v, (v, j<i) and itself.
        Returns (Z[T, V], g[T], Dall[T, k, V]); the cache is written exactly as in `verify`."""
        c, n, t_rows = self.cfg, self.n, self.T
        x = self.m.embed(tok)                       # rows 0..T-1 are tree rows; pseudo rows appended
        owner = list(range(t_rows))                 # tree node each row belongs to
        step = [0] * t_rows                         # 0 = real row, i>=1 = pseudo step
        for layer in range(c.n_layers):
            for i, t in enumerate(c.transfer_layers):
                if t == layer:
                    new = linear(x[:t_rows], self.m.w.w_transfer[i])
                    x = np.concatenate([x, new], axis=0)
                    owner += list(range(t_rows))
                    step += [i + 1] * t_rows
            r = x.shape[0]
            pos = np.array([n + self.depth[owner[a]] + step[a] for a in range(r)])
            vis_new = np.zeros((r, r), dtype=bool)
            for a in range(r):
                for b in range(r):
                    if step[b] == 0:                # real tree row: visible to a if ancestor-or-self of a's owner
                        vis_new[a, b] = self.anc[owner[a], owner[b]]
                    else:                           # pseudo row: same owner, earlier-or-same step
                        vis_new[a, b] = owner[a] == owner[b] and 0 < step[b] <= step[a]
            vis_old = np.ones((r, n), dtype=bool)
            x, k, v = self.m.block(layer, x, pos, self.K[layer][:n], self.V[layer][:n], vis_old, vis_new)
            self.K[layer][n:n + t_rows], self.V[layer][n:n + t_rows] = k[:t_rows], v[:t_rows]
        z_all = self.m.logits(x)
        z = z_all[:t_rows]
        d_all = np.zeros((t_rows, c.k, c.vocab))
        for a in range(t_rows, x.shape[0]):
            d_all[owner[a], step[a] - 1] = z_all[a]
        return z, [int(j) for j in np.argmax(z, axis=1)], d_all
