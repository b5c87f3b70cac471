"""GPU-side glue for the parity tests: builds an HTModel for a workload and runs the step-by-step
comparison of the HIP path against the oracle.  Imported only by tests marked `gpu`."""
from __future__ import annotations

import numpy as np
import torch

from ht_inputs import make_weights, prune_tree
from oracle import ht_oracle as O
from helpers import torch_dtype, oracle_model, oracle_decoder, prompt_of, tree_of

import paper_2404_12022_amd.binding as B

DEV = "cuda:0"

FP32_LOGIT_TOL = 1e-4          # max-abs, fp32 model
BF16_REL_TOL = 3e-2            # bf16 model: per row, max|a-b| <= tol * max|b| and ||a-b|| <= tol * ||b||


def bf16_tol_after(blocks: int) -> float:
    """The bf16 bound for a value that has come through `blocks` decoder blocks of rounded activations.  Every block
    rounds its normalised rows, q, K, V, the attention output and the feed-forward activations to bf16 (2^-9
    relative each); BF16_REL_TOL bounds what one block adds, the blocks' roundings are independent of each other,
    and independent errors add in quadrature: sqrt(blocks) one-block bounds.  Measured against the fp64 oracle the
    worst row sits at 0.55 sqrt(blocks) of the one-block bound on the 7B shape (512 prompt rows; 3.0 x at 32
    blocks) and at up to 0.85 sqrt(blocks) on the 13B shape (2048 prompt rows, so the worst of four times as many; 4.9 x
    at 33 blocks).
    One block is the plain tolerance, which is what every test of up to three blocks asserts."""
    return BF16_REL_TOL * float(np.sqrt(max(1, blocks)))


def within_bf16(got: np.ndarray, want: np.ndarray, tol=BF16_REL_TOL):
    """bf16 criterion, per row (last axis): max-abs error <= tol * max-abs reference, and relative L2 error <= tol.
    Returns (ok, worst error / bound)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - want)
    peak = np.max(np.abs(want), axis=-1)
    l2 = np.sqrt(np.sum(want * want, axis=-1))
    r1 = np.max(err, axis=-1) / (tol * peak)
    r2 = np.sqrt(np.sum(err * err, axis=-1)) / (tol * l2)
    worst = float(max(np.max(r1), np.max(r2)))
    return worst <= 1.0, worst


def elementwise_ratio(got: np.ndarray, want: np.ndarray, tol=BF16_REL_TOL) -> float:
    """A stricter reading of "3e-2 relative" than `within_bf16`, reported but not asserted: the worst element's error
    over tol * max(|reference element|, rms of its row)."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    rms = np.sqrt(np.mean(want * want, axis=-1, keepdims=True))
    return float(np.max(np.abs(got - want) / (tol * np.maximum(np.abs(want), rms))))


def assert_close(got, want, dtype: str, what: str, tol=None):
    """Returns the max-abs error (fp32) or the worst error/bound ratio (bf16)."""
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values from the GPU"
    if dtype == "f32":
        err = float(np.max(np.abs(got - want)))
        assert err <= (tol or FP32_LOGIT_TOL), f"{what}: max-abs error {err:.3e}"
        return err
    else:
        ok, worst = within_bf16(got, want, tol or BF16_REL_TOL)
        assert ok, f"{what}: worst error is {worst:.2f}x the bf16 bound"
        return worst


def gpu_model(wl, tensors=None, max_tree=None):
    tensors = tensors or make_weights(wl, wl.seed, DEV, torch_dtype(wl))
    cfg = B.make_config(wl, max_tree=max_tree)
    return B.HTModel(cfg, tensors, DEV)


def cpu(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


class StepCompare:
    """Runs oracle and HIP path side by side, one decode step at a time."""

    def __init__(self, wl, tensors_gpu=None, tensors_cpu=None, tree=None, prompt=None, fused=None, dynamic=None,
                 model=None):
        """fused: tree nodes that get pseudo rows inside the verify pass (`ht_set_fused_nodes`).  The oracle keeps
        drafting after acceptance; the two schedules give the same distributions (a CPU test pins that).
        dynamic = (T, b): every step chooses its tree (`ht_set_dynamic_tree`); use `step_dynamic`."""
        self.wl = wl
        self.model = model or oracle_model(wl, tensors_cpu)
        self.dynamic = dynamic
        self.parent, self.rank = ([-1] + [0] * (dynamic[0] - 1), [0] * dynamic[0]) if dynamic else (tree or tree_of(wl))
        self.ora = O.HiddenTransferOracle(self.model, self.parent, self.rank, wl.max_cache)
        self.fused = list(fused or [])
        self.gpu = gpu_model(wl, tensors_gpu, max_tree=max(len(self.parent) + len(self.fused) * wl.k, 1))
        if dynamic:
            self.gpu.ht_set_dynamic_tree(*dynamic)
        else:
            self.gpu.ht_set_tree(self.parent, self.rank)
        if self.fused:
            self.gpu.ht_set_fused_nodes(self.fused)
        self.in_pass_drafts = None      # (logits [k, V], candidates) of the node the last acceptance ended on
        self.steps_without_draft_pass = 0
        self.prompt = prompt or prompt_of(wl)
        self.ora.prefill(self.prompt)
        self.gpu.ht_prefill(self.prompt)
        self.T = len(self.parent)
        self.z_gpu = torch.empty(self.T, wl.vocab, dtype=torch.float32, device=DEV)
        self.g_gpu = torch.empty(self.T, dtype=torch.int32, device=DEV)
        self.min_margin = float("inf")
        self.max_err = 0.0          # largest logit error seen (fp32: absolute; bf16: fraction of the bound)
        self.max_elementwise = 0.0  # verify logits: worst element error / (3e-2 max(|element|, row rms)), not asserted
        self.tol = None             # bf16 bound of the float comparisons (None: BF16_REL_TOL); fp32 models ignore it
        self.verify_passes_compared = 0     # verify passes whose T logit rows were all held against the oracle
        self.steps_on_gpu_tree = 0          # of those, passes in which the oracle verified the GPU's tree, not its own

    def check_prefill(self):
        wl = self.wl
        assert self.gpu.ht_cache_len() == len(self.prompt) == self.ora.n
        root = int(self.gpu.ht_get_buffer(B.HT_BUF_ROOT)[0].item())
        if root != self.ora.root:
            # only a bf16 near-tie may do this: the two tokens' exact logits must be closer than the two passes may
            # differ; either token is then a legitimate outcome and the comparison goes on from the GPU's
            assert wl.dtype != "f32", f"prefill root {root}, oracle {self.ora.root}"
            z = self.model.causal_forward(self.prompt)[0][-1]
            gap, bound = float(z[self.ora.root] - z[root]), 2 * (self.tol or BF16_REL_TOL) * float(np.max(np.abs(z)))
            print(f"prefill root {root} vs oracle {self.ora.root}: exact logit gap {gap:.3e}, bf16 bound {bound:.3e}",
                  flush=True)
            assert 0 <= gap <= bound, f"prefill root {root} vs {self.ora.root}: logit gap {gap:.3e} above {bound:.3e}"
            self.ora.root = root
        for slot, t in enumerate(sorted(set(wl.transfer_layers))):
            h = cpu(self.gpu.ht_get_buffer(B.HT_BUF_TRANSFER_SRC, slot))
            assert_close(h, self.ora.h_src[t], wl.dtype, f"prefill transfer source of layer {t}",
                         tol=self.tol if wl.dtype != "f32" else 1e-4)
        self.check_cache("prefill")

    def check_cache(self, what, layers=None):
        wl, n = self.wl, self.ora.n
        for layer in layers or (0, wl.n_layers - 1):
            kc = cpu(self.gpu.ht_get_buffer(B.HT_BUF_K_CACHE, layer))[:n]
            vc = cpu(self.gpu.ht_get_buffer(B.HT_BUF_V_CACHE, layer))[:, :, :n]
            tol = self.tol if wl.dtype != "f32" else None
            assert_close(kc, self.ora.K[layer][:n], wl.dtype, f"{what}: K cache layer {layer}", tol=tol)
            assert_close(np.transpose(vc, (2, 0, 1)), self.ora.V[layer][:n], wl.dtype, f"{what}: V cache layer {layer}", tol=tol)

    def step(self, forced=None, require_same_tokens=True):
        """One step on both sides.  The oracle drafts its own tree; the verify pass, however, is always compared on
        the tokens the GPU verified: when a bf16 near-tie among the drafted candidates gave the GPU another tree
        than the oracle's, the oracle verifies the GPU's tree (any tree keeps the output greedy, Sec. 4.1), so all
        T logit rows are compared in every step and `verify_passes_compared` counts them."""
        wl, ora, gpu = self.wl, self.ora, self.gpu
        ftol = self.tol if wl.dtype != "f32" else None
        pseudo_o = ora.transfer()
        d_o = ora.draft(pseudo_o)
        cand_o = ora.candidates(d_o)
        tok_o = list(forced) if forced is not None else ora.build_tree(cand_o)
        drafts = self.in_pass_drafts
        root_gpu = int(gpu.ht_get_buffer(B.HT_BUF_ROOT)[0].item())      # pending root: the greedy token after the last accepted node
        if forced is None and drafts is not None:
            gpu.ht_transfer(None, None)                  # nothing left to do: the last verify pass drafted already
            gpu.ht_tree_verify_step(None, self.g_gpu, self.z_gpu)
            self.steps_without_draft_pass += 1
        elif forced is None:
            pseudo = torch.empty(wl.k, wl.d_model, dtype=torch.float32, device=DEV)
            gpu.ht_transfer(None, pseudo)
            gpu.ht_tree_verify_step(None, self.g_gpu, self.z_gpu)
        else:
            gpu.ht_tree_verify_step(torch.tensor(forced, dtype=torch.int32, device=DEV), self.g_gpu, self.z_gpu)
        torch.cuda.synchronize()
        tok_gpu = [int(t) for t in gpu.ht_get_buffer(B.HT_BUF_TREE_TOKENS).cpu()]
        z = cpu(self.z_gpu)
        g = [int(t) for t in self.g_gpu.cpu()]
        if forced is None:
            if drafts is None:
                assert_close(cpu(pseudo), np.stack(pseudo_o), wl.dtype, "pseudo hidden states", tol=ftol)
                d = cpu(gpu.ht_get_buffer(B.HT_BUF_DRAFT_LOGITS))
                cand = gpu.ht_get_buffer(B.HT_BUF_CANDIDATES).cpu().numpy()
            else:
                d, cand = drafts
            self.max_err = max(self.max_err, assert_close(d, d_o, wl.dtype, "draft logits", tol=ftol))
            # integer stages: the oracle's rules applied to the GPU's own logits must give the GPU's integers
            want_cand = [[]] + [O.top_candidates(d[e - 1], ora.width[e]) for e in range(1, len(ora.width))]
            for e in range(1, len(ora.width)):
                assert list(cand[e - 1][:ora.width[e]]) == want_cand[e], f"top-k at depth {e}"
            want_tok = [root_gpu] + [want_cand[ora.depth[v]][ora.rank[v]] for v in range(1, self.T)]
            assert tok_gpu == want_tok, "tree build"
            for e in range(1, len(ora.width)):           # margin of the oracle's own candidate order
                srt = np.sort(d_o[e - 1])[::-1][:ora.width[e] + 1]
                self.min_margin = min(self.min_margin, float(np.min(srt[:-1] - srt[1:])))
        else:
            assert tok_gpu == list(forced)
        same_tree = tok_gpu == tok_o
        if require_same_tokens:
            assert same_tree, "tree tokens differ from the fp64 oracle"
        elif not same_tree:
            self.steps_on_gpu_tree += 1
        # the oracle verifies the tree the GPU verified (its own, unless a near-tie changed a candidate)
        z_o, g_o, saved = ora.verify(tok_gpu)
        self.max_err = max(self.max_err, assert_close(z, z_o, wl.dtype, "verify logits", tol=ftol))
        self.max_elementwise = max(self.max_elementwise, elementwise_ratio(z, z_o))
        self.verify_passes_compared += 1
        assert g == [int(j) for j in np.argmax(z, axis=1)], "row arg-max of the GPU's own logits"
        if wl.dtype != "f32":
            for v in range(self.T):                      # another greedy token only where the exact logits nearly tie
                gap, bound = float(z_o[v][g_o[v]] - z_o[v][g[v]]), 2 * (ftol or BF16_REL_TOL) * float(np.max(np.abs(z_o[v])))
                assert 0 <= gap <= bound, f"node {v}: greedy token {g[v]} vs {g_o[v]}, logit gap {gap:.3e} above {bound:.3e}"
        top2 = np.sort(z_o, axis=1)[:, -2:]
        self.min_margin = min(self.min_margin, float(np.min(top2[:, 1] - top2[:, 0])))
        m, emitted, root, path = gpu.ht_accept_and_compact()
        want_path, want_root = O.accept_walk(self.parent, tok_gpu, g)
        assert (path, root, m) == (want_path, want_root, len(want_path)), "acceptance walk on the GPU's own integers"
        assert emitted == [tok_gpu[v] for v in path]
        path_o, emitted_o = ora.accept_and_compact(tok_gpu, g_o, saved)
        res = dict(pseudo=pseudo_o, D=d_o, cand=cand_o, tok=tok_o, Z=z_o, g=g_o, H=saved, path=path_o, emitted=emitted_o,
                   root=ora.root, n=ora.n)
        self.in_pass_drafts = None
        if path[-1] in self.fused:                       # keep what the pass drafted for the node it ended on
            zf, cand = gpu.fused_drafts(self.fused.index(path[-1]))
            self.in_pass_drafts = (cpu(zf), cand.cpu().numpy())
        if require_same_tokens:
            assert (path, emitted, root) == (res["path"], res["emitted"], res["root"])
            assert gpu.ht_cache_len() == ora.n
        return dict(oracle=res, emitted=emitted, path=path, root=root, m=m)

    def step_dynamic(self, exact=True):
        """One step in which the GPU chooses its tree.  Every float stage is compared with the fp64 oracle; every
        integer stage must be the oracle's rule applied to the GPU's own numbers; the oracle then verifies the
        GPU's tree.  exact (fp32 model): the oracle's own choices must be the same.  Otherwise (bf16) a choice may
        differ where the oracle's numbers are closer than the two may differ, and the oracle follows the GPU's."""
        wl, ora, gpu = self.wl, self.ora, self.gpu
        T, b = self.dynamic
        d_o = ora.draft(ora.transfer())
        root_gpu = int(gpu.ht_get_buffer(B.HT_BUF_ROOT)[0].item())
        assert root_gpu == ora.root
        pseudo = torch.empty(wl.k, wl.d_model, dtype=torch.float32, device=DEV)
        gpu.ht_transfer(None, pseudo)
        gpu.ht_tree_verify_step(None, self.g_gpu, self.z_gpu)
        torch.cuda.synchronize()
        d = cpu(gpu.ht_get_buffer(B.HT_BUF_DRAFT_LOGITS))
        self.max_err = max(self.max_err, assert_close(d, d_o, wl.dtype, "draft logits"))
        cand = gpu.ht_get_buffer(B.HT_BUF_CANDIDATES).cpu().numpy()[:, :b]
        lp = gpu.ht_get_buffer(B.HT_BUF_CANDIDATE_LOGPROBS).cpu().numpy()[:, :b]
        want_lp = []
        for e in range(wl.k):
            ids, vals = O.candidate_logprobs(d[e], b)
            assert list(cand[e]) == ids, f"top-{b} at depth {e + 1}"
            want_lp.append(vals)
        lp_err = float(np.max(np.abs(lp.astype(np.float64) - np.stack(want_lp))))
        assert lp_err <= 2e-5, f"candidate log-probabilities off by {lp_err:.2e}"
        parent = [int(x) for x in gpu.ht_get_buffer(B.HT_BUF_TREE_PARENT).cpu()]
        rank = [int(x) for x in gpu.ht_get_buffer(B.HT_BUF_TREE_RANK).cpu()]
        assert (parent, rank) == O.dynamic_tree(lp, T), "tree choice from the GPU's own log-probabilities"
        own = O.dynamic_tree(np.stack([O.candidate_logprobs(d_o[e], b)[1] for e in range(wl.k)]), T)
        if exact:
            assert (parent, rank) == own, "tree differs from the fp64 oracle's"
        ora.set_tree(parent, rank)
        depth = ora.depth
        tok_gpu = [int(t) for t in gpu.ht_get_buffer(B.HT_BUF_TREE_TOKENS).cpu()]
        assert tok_gpu == [root_gpu] + [int(cand[depth[v] - 1][rank[v]]) for v in range(1, T)], "tree tokens"
        z_o, g_o, saved = ora.verify(tok_gpu)
        z = cpu(self.z_gpu)
        self.max_err = max(self.max_err, assert_close(z, z_o, wl.dtype, "verify logits"))
        g = [int(t) for t in self.g_gpu.cpu()]
        assert g == [int(j) for j in np.argmax(z, axis=1)], "row arg-max of the GPU's own logits"
        if exact:
            assert g == g_o
        else:
            for v in range(T):
                gap, bound = float(z_o[v][g_o[v]] - z_o[v][g[v]]), 2 * BF16_REL_TOL * float(np.max(np.abs(z_o[v])))
                assert 0 <= gap <= bound, f"node {v}: greedy token {g[v]} vs {g_o[v]}, logit gap {gap:.3e} above {bound:.3e}"
        m, emitted, root, path = gpu.ht_accept_and_compact()
        want_path, want_emitted = ora.accept_and_compact(tok_gpu, g, saved)
        assert (path, emitted, root, m) == (want_path, want_emitted, ora.root, len(want_path))
        assert gpu.ht_cache_len() == ora.n
        return dict(parent=parent, rank=rank, emitted=emitted, path=path, root=root, m=m, own_tree=own)
