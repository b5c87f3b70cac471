"""ctypes binding of libht.so: the same entry points as include/ht.h, argument marshalling only.

`HTModel` is a convenience holder that keeps the torch tensors (weights, workspace) alive and turns
them into pointers; it performs no arithmetic.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libht.so")

HT_OK, HT_EINVAL, HT_ECAPACITY, HT_ETREE, HT_ESTATE, HT_EHIP, HT_EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
HT_F32, HT_BF16 = 0, 1
HT_MAX_TRANSFER, HT_MAX_TREE, HT_MAX_ROWS, HT_MAX_TOPK = 8, 128, 256, 64
HT_MAX_LOOP_STEPS = 64
(HT_BUF_DRAFT_LOGITS, HT_BUF_CANDIDATES, HT_BUF_TREE_TOKENS, HT_BUF_SAVED_HIDDEN, HT_BUF_TRANSFER_SRC,
 HT_BUF_K_CACHE, HT_BUF_V_CACHE, HT_BUF_PSEUDO, HT_BUF_ROOT, HT_BUF_FUSED_DRAFT_LOGITS,
 HT_BUF_FUSED_CANDIDATES, HT_BUF_CANDIDATE_LOGPROBS, HT_BUF_TREE_PARENT, HT_BUF_TREE_RANK) = range(14)

EXPORTS = [
    "ht_workspace_bytes", "ht_init_model", "ht_free_model", "ht_set_tree", "ht_prefill", "ht_transfer",
    "ht_tree_verify_step", "ht_accept_and_compact", "ht_cache_len", "ht_last_error", "ht_get_buffer",
    "ht_tree_attention_scratch_bytes", "ht_tree_attention", "ht_padded_rows", "ht_skinny_gemm_scratch_bytes",
    "ht_skinny_gemm", "ht_weight_pack_bytes", "ht_weight_pack", "ht_skinny_gemm_packed", "ht_load_layer",
    "ht_load_lm_head", "ht_set_fused_nodes", "ht_stream_read_probe", "ht_mfma_rate_probe", "ht_decode_steps",
    "ht_gate_up_pack", "ht_gate_up_silu_packed", "ht_set_dynamic_tree", "ht_candidate_logprobs", "ht_dynamic_tree",
    "ht_training_forward", "ht_kl_divergence_rows", "ht_skinny_gemm_packed_noalloc",
    "ht_training_workspace_bytes", "ht_training_forward_batched",
]


class ht_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + [
        ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32), ("k", C.c_int32),
        ("transfer_layer", C.c_int32 * HT_MAX_TRANSFER), ("max_cache", C.c_int32), ("max_tree", C.c_int32)]


_PP = C.POINTER(C.c_void_p)


class ht_weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("attn_norm", _PP), ("wq", _PP), ("wk", _PP), ("wv", _PP), ("wo", _PP), ("ffn_norm", _PP),
                ("w_gate", _PP), ("w_up", _PP), ("w_down", _PP), ("w_transfer", _PP)]


class HTError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libht error {code}: {message}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2404_12022_amd.build); "
                          "there is no fallback path")
    # torch first: the library and torch must share one HIP runtime, and the one torch loads has to be in the
    # process before libht.so resolves its own dependency (loaded the other way round, the library's runtime
    # finds no device)
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    i32p, f32p, vp, sz = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p, C.c_size_t
    sig = {
        "ht_workspace_bytes": (C.c_int, [C.POINTER(ht_config), C.POINTER(sz)]),
        "ht_init_model": (C.c_int, [C.POINTER(ht_config), C.POINTER(ht_weights), vp, sz, vp, C.POINTER(vp)]),
        "ht_free_model": (C.c_int, [vp]),
        "ht_set_tree": (C.c_int, [vp, C.c_int32, i32p, i32p, vp]),
        "ht_set_fused_nodes": (C.c_int, [vp, C.c_int32, i32p, vp]),
        "ht_set_dynamic_tree": (C.c_int, [vp, C.c_int32, C.c_int32, vp]),
        "ht_kl_divergence_rows": (C.c_int, [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp]),
        "ht_training_forward": (C.c_int, [vp, C.c_int32, i32p, C.c_int32, f32p, C.POINTER(C.c_double), vp, vp, vp]),
        "ht_training_workspace_bytes": (C.c_int, [C.POINTER(ht_config), C.c_int32, C.POINTER(sz)]),
        "ht_training_forward_batched": (C.c_int, [vp, C.c_int32, i32p, C.c_int32, f32p, C.POINTER(C.c_double), vp, vp, vp, sz,
                                                  vp]),
        "ht_candidate_logprobs": (C.c_int, [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]),
        "ht_dynamic_tree": (C.c_int, [vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp, vp, vp, vp]),
        "ht_stream_read_probe": (C.c_int, [vp, sz, vp, C.POINTER(sz), vp]),
        "ht_mfma_rate_probe": (C.c_int, [C.c_int32, C.c_int32, vp, C.POINTER(C.c_double), vp]),
        "ht_prefill": (C.c_int, [vp, i32p, C.c_int32, vp]),
        "ht_transfer": (C.c_int, [vp, vp, vp, vp]),
        "ht_tree_verify_step": (C.c_int, [vp, vp, vp, vp, vp]),
        "ht_accept_and_compact": (C.c_int, [vp, i32p, i32p, i32p, i32p, vp]),
        "ht_gate_up_pack": (C.c_int, [vp, vp, C.c_int32, C.c_int32, vp, vp]),
        "ht_gate_up_silu_packed": (C.c_int, [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]),
        "ht_decode_steps": (C.c_int, [vp, C.c_int32, i32p, i32p, i32p, vp]),
        "ht_cache_len": (C.c_int32, [vp]),
        "ht_last_error": (C.c_char_p, []),
        "ht_get_buffer": (C.c_int, [vp, C.c_int32, C.c_int32, C.POINTER(vp), C.POINTER(sz)]),
        "ht_tree_attention_scratch_bytes": (sz, [C.c_int32, C.c_int32, C.c_int32]),
        "ht_tree_attention": (C.c_int, [vp, vp, vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, i32p, C.c_int32, C.c_int32,
                                        C.c_int32, C.c_int32, C.c_float, vp, vp, sz, vp]),
        "ht_padded_rows": (C.c_int32, [C.c_int32]),
        "ht_skinny_gemm_scratch_bytes": (sz, [C.c_int32, C.c_int32, C.c_int32]),
        "ht_skinny_gemm": (C.c_int, [vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp, sz, vp]),
        "ht_load_layer": (C.c_int, [vp, C.c_int32, vp, vp, vp, vp, vp, vp, vp, vp]),
        "ht_load_lm_head": (C.c_int, [vp, vp, vp]),
        "ht_weight_pack_bytes": (sz, [C.c_int32, C.c_int32]),
        "ht_weight_pack": (C.c_int, [vp, C.c_int32, C.c_int32, vp, vp]),
        "ht_skinny_gemm_packed": (C.c_int, [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp, sz, vp]),
        "ht_skinny_gemm_packed_noalloc": (C.c_int, [vp, vp, C.c_int32, C.c_int32, C.c_int32, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


lib = _load()


def _check(rc: int) -> None:
    if rc != HT_OK:
        raise HTError(rc, lib.ht_last_error().decode())


def _i32(seq: Sequence[int]):
    return (C.c_int32 * len(seq))(*[int(v) for v in seq])


def _stream_ptr(stream=None) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


# ------------------------------------------------------------------ thin wrappers, same names as the ABI
def ht_last_error() -> str:
    return lib.ht_last_error().decode()


def ht_padded_rows(m: int) -> int:
    return lib.ht_padded_rows(m)


def ht_workspace_bytes(cfg: ht_config) -> int:
    out = C.c_size_t(0)
    _check(lib.ht_workspace_bytes(C.byref(cfg), C.byref(out)))
    return out.value


def ht_tree_attention_scratch_bytes(T: int, Hq: int, hd: int) -> int:
    return lib.ht_tree_attention_scratch_bytes(T, Hq, hd)


def ht_tree_attention(q, k_new, v_new, k_cache, v_cache, cap, n, T, parent, Hq, Hkv, hd, dtype, rope_base, out, scratch,
                      stream=None) -> None:
    _check(lib.ht_tree_attention(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache), cap, n, T,
                                 None if parent is None else _i32(parent), Hq, Hkv, hd, dtype, rope_base, _ptr(out),
                                 _ptr(scratch),
                                 scratch.numel() * scratch.element_size(), _stream_ptr(stream)))


def ht_skinny_gemm_scratch_bytes(M: int, N: int, K: int) -> int:
    return lib.ht_skinny_gemm_scratch_bytes(M, N, K)


def ht_skinny_gemm(a, w, M, N, K, dtype, out, scratch=None, stream=None) -> None:
    sb = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib.ht_skinny_gemm(_ptr(a), _ptr(w), M, N, K, dtype, _ptr(out), _ptr(scratch), sb, _stream_ptr(stream)))


def ht_weight_pack_bytes(N: int, K: int) -> int:
    return lib.ht_weight_pack_bytes(N, K)


def ht_weight_pack(w, N, K, packed, stream=None) -> None:
    _check(lib.ht_weight_pack(_ptr(w), N, K, _ptr(packed), _stream_ptr(stream)))


def ht_skinny_gemm_packed(a, packed, M, N, K, out, scratch=None, stream=None) -> None:
    sb = 0 if scratch is None else scratch.numel() * scratch.element_size()
    _check(lib.ht_skinny_gemm_packed(_ptr(a), _ptr(packed), M, N, K, _ptr(out), _ptr(scratch), sb, _stream_ptr(stream)))


HT_NOALLOC_SCRATCH_BYTES = 16 << 20


def ht_skinny_gemm_packed_noalloc(a, packed, M, N, K, out, stream=None) -> None:
    _check(lib.ht_skinny_gemm_packed_noalloc(_ptr(a), _ptr(packed), M, N, K, _ptr(out), _stream_ptr(stream)))


def ht_gate_up_pack(w_gate, w_up, f, K, packed, stream=None) -> None:
    _check(lib.ht_gate_up_pack(_ptr(w_gate), _ptr(w_up), f, K, _ptr(packed), _stream_ptr(stream)))


def ht_gate_up_silu_packed(a, packed, M, f, K, act_out, stream=None) -> None:
    _check(lib.ht_gate_up_silu_packed(_ptr(a), _ptr(packed), M, f, K, _ptr(act_out), _stream_ptr(stream)))


def ht_kl_divergence_rows(z, row_a, row_b, pairs, kl, stream=None) -> None:
    """z [rows, V] float32, kl [pairs] float32 (device tensors): kl[p] = KL(softmax z[row_a + p] || softmax z[row_b + p])."""
    _check(lib.ht_kl_divergence_rows(_ptr(z), row_a, row_b, pairs, z.shape[1], _ptr(kl), _stream_ptr(stream)))


def ht_candidate_logprobs(d, cand, b, lp, stream=None) -> None:
    """d [rows, V] float32, cand [rows, HT_MAX_TOPK] int32, lp [rows, HT_MAX_TOPK] float32 (device tensors)."""
    _check(lib.ht_candidate_logprobs(_ptr(d), _ptr(cand), d.shape[0], b, d.shape[1], _ptr(lp), _stream_ptr(stream)))


def ht_dynamic_tree(lp, cand, root, k, b, T, parent, depth, rank, anc, tokens, stream=None) -> None:
    """All arguments but k, b, T are device tensors: lp, cand [k, HT_MAX_TOPK], root [1]; outputs parent, depth, rank,
    tokens [T] int32 and anc [T, HT_MAX_ROWS // 64] int64."""
    _check(lib.ht_dynamic_tree(_ptr(lp), _ptr(cand), _ptr(root), k, b, T, _ptr(parent), _ptr(depth), _ptr(rank),
                               _ptr(anc), _ptr(tokens), _stream_ptr(stream)))


def ht_stream_read_probe(buf, sink, stream=None) -> int:
    """One streaming pass over the tensor `buf`; returns the bytes read."""
    got = C.c_size_t(0)
    _check(lib.ht_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), C.byref(got),
                                    _stream_ptr(stream)))
    return got.value


def ht_mfma_rate_probe(form: int, iters: int, sink, stream=None) -> float:
    """One launch of the matrix-core probe (form 0: 16x16x32, 1: 32x32x16, + 2: hashed operand bits); returns its
    floating-point operations."""
    got = C.c_double(0.0)
    _check(lib.ht_mfma_rate_probe(form, iters, _ptr(sink), C.byref(got), _stream_ptr(stream)))
    return got.value


def make_config(shape, max_cache: Optional[int] = None, max_tree: Optional[int] = None) -> ht_config:
    """ht_config from any object with the Workload attributes."""
    cfg = ht_config()
    for name in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "k"):
        setattr(cfg, name, int(getattr(shape, name)))
    cfg.rms_eps, cfg.rope_base = float(shape.rms_eps), float(shape.rope_base)
    cfg.dtype = HT_F32 if shape.dtype == "f32" else HT_BF16
    for i, t in enumerate(shape.transfer_layers):
        cfg.transfer_layer[i] = int(t)
    cfg.max_cache = int(max_cache if max_cache is not None else shape.max_cache)
    cfg.max_tree = int(max_tree if max_tree is not None else shape.tree_size)
    return cfg


class HTModel:
    """Owns the workspace tensor and the pointer tables for one ht_model handle."""

    def __init__(self, cfg: ht_config, weights: Dict[str, object], device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.weights = weights                      # keep the tensors alive
        self.device = torch.device(device)
        L, k = cfg.n_layers, cfg.k
        w = ht_weights()
        w.tok_emb, w.final_norm = (weights[n].data_ptr() for n in ("tok_emb", "final_norm"))
        w.lm_head = _ptr(weights.get("lm_head"))           # None: supplied later through ht_load_lm_head
        self._tables = {}
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            arr = (C.c_void_p * L)(*[_ptr(weights[name][l]) for l in range(L)])   # None: ht_load_layer later
            self._tables[name] = arr
            setattr(w, name, C.cast(arr, _PP))
        arr = (C.c_void_p * k)(*[weights["w_transfer"][i].data_ptr() for i in range(k)])
        self._tables["w_transfer"] = arr
        w.w_transfer = C.cast(arr, _PP)
        nbytes = ht_workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        handle = C.c_void_p()
        _check(lib.ht_init_model(C.byref(cfg), C.byref(w), self.workspace.data_ptr(), nbytes, _stream_ptr(stream),
                                 C.byref(handle)))
        self.handle = handle
        self.T = 0

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib.ht_free_model(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the ABI calls
    def ht_load_layer(self, layer: int, tensors: Dict[str, object], stream=None) -> None:
        _check(lib.ht_load_layer(self.handle, layer, *[tensors[n].data_ptr() for n in
                                                       ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")],
                                 _stream_ptr(stream)))

    def ht_load_lm_head(self, lm_head, stream=None) -> None:
        _check(lib.ht_load_lm_head(self.handle, lm_head.data_ptr(), _stream_ptr(stream)))

    def ht_set_tree(self, parent: Sequence[int], rank: Sequence[int], stream=None) -> None:
        _check(lib.ht_set_tree(self.handle, len(parent), _i32(parent), _i32(rank), _stream_ptr(stream)))
        self.T = len(parent)
        self.fused = []

    def ht_set_dynamic_tree(self, T: int, b: int, stream=None) -> None:
        _check(lib.ht_set_dynamic_tree(self.handle, T, b, _stream_ptr(stream)))
        self.T = T
        self.fused = []

    def ht_training_forward(self, step: int, tokens: Sequence[int], logits_hidden=None, logits_pseudo=None, stream=None):
        """Returns (kl list of n - step - 1 floats, loss).  logits_hidden [n, vocab], logits_pseudo [n - step + 1, vocab]:
        optional float32 device tensors that receive the logits."""
        n = len(tokens)
        kl = (C.c_float * max(n - step - 1, 1))()
        loss = C.c_double(0.0)
        _check(lib.ht_training_forward(self.handle, step, _i32(tokens), n, kl, C.byref(loss),
                                       _ptr(logits_hidden) if logits_hidden is not None else None,
                                       _ptr(logits_pseudo) if logits_pseudo is not None else None, _stream_ptr(stream)))
        return [float(v) for v in kl[:max(n - step - 1, 0)]], loss.value

    def ht_training_forward_batched(self, step: int, tokens: Sequence[int], logits_hidden=None, logits_pseudo=None,
                                    workspace=None, stream=None):
        """`ht_training_forward` with all positions in one pass per block.  workspace: a uint8 device tensor of at least
        `ht_training_workspace_bytes` bytes (allocated here when None).  Returns (kl list, loss)."""
        n = len(tokens)
        if workspace is None:
            need = C.c_size_t(0)
            _check(lib.ht_training_workspace_bytes(C.byref(self.cfg), n, C.byref(need)))
            workspace = self.torch.empty(need.value, dtype=self.torch.uint8, device=self.device)
        kl = (C.c_float * max(n - step - 1, 1))()
        loss = C.c_double(0.0)
        _check(lib.ht_training_forward_batched(self.handle, step, _i32(tokens), n, kl, C.byref(loss),
                                               _ptr(logits_hidden) if logits_hidden is not None else None,
                                               _ptr(logits_pseudo) if logits_pseudo is not None else None,
                                               _ptr(workspace), workspace.numel(), _stream_ptr(stream)))
        return [float(v) for v in kl[:max(n - step - 1, 0)]], loss.value

    def ht_set_fused_nodes(self, nodes: Sequence[int], stream=None) -> None:
        _check(lib.ht_set_fused_nodes(self.handle, len(nodes), _i32(nodes) if len(nodes) else None, _stream_ptr(stream)))
        self.fused = list(nodes)

    def ht_prefill(self, tokens: Sequence[int], stream=None) -> None:
        _check(lib.ht_prefill(self.handle, _i32(tokens), len(tokens), _stream_ptr(stream)))

    def ht_transfer(self, h_src=None, pseudo_out=None, stream=None) -> None:
        _check(lib.ht_transfer(self.handle, _ptr(h_src), _ptr(pseudo_out), _stream_ptr(stream)))

    def ht_tree_verify_step(self, tree_tokens=None, argmax_out=None, logits_out=None, stream=None) -> None:
        _check(lib.ht_tree_verify_step(self.handle, _ptr(tree_tokens), _ptr(argmax_out), _ptr(logits_out),
                                       _stream_ptr(stream)))

    def ht_accept_and_compact(self, stream=None):
        k1 = self.cfg.k + 1
        m, root = C.c_int32(0), C.c_int32(0)
        toks, path = (C.c_int32 * k1)(), (C.c_int32 * k1)()
        _check(lib.ht_accept_and_compact(self.handle, C.byref(m), toks, C.byref(root), path, _stream_ptr(stream)))
        return m.value, list(toks[:m.value]), root.value, list(path[:m.value])

    def ht_decode_steps(self, steps: int, stream=None):
        """(accepted count per step, emitted tokens of every step as one list, pending root)."""
        counts = (C.c_int32 * steps)()
        toks = (C.c_int32 * (steps * (self.cfg.k + 1)))()
        root = C.c_int32(0)
        _check(lib.ht_decode_steps(self.handle, steps, counts, toks, C.byref(root), _stream_ptr(stream)))
        counts = list(counts)
        return counts, list(toks[:sum(counts)]), root.value

    def decode(self, max_new_tokens: int, stream=None):
        """Calls transfer / verify / accept until at least `max_new_tokens` tokens are out or the cache is full
        (after `ht_set_tree` and `ht_prefill`).  Returns the emitted tokens: the greedy continuation of the prompt.
        A loop over the ABI calls and nothing else."""
        rows = max(self.T + len(getattr(self, "fused", [])) * self.cfg.k, self.cfg.k)
        out = []
        while len(out) < max_new_tokens and self.ht_cache_len() + rows <= self.cfg.max_cache:
            self.ht_transfer(None, None, stream)
            self.ht_tree_verify_step(None, None, None, stream)
            _, emitted, _, _ = self.ht_accept_and_compact(stream)
            out += emitted
        return out

    def fused_drafts(self, f: int):
        """(draft logits [k, vocab], candidates [k, HT_MAX_TOPK]) that the last verify pass produced for fused node
        number f.  The pass holds pseudo rows in the order they joined: transfer-layer slot by slot, node by node,
        step by step."""
        c = self.cfg
        layers = list(c.transfer_layer[:c.k])
        firsts = [i for i in range(c.k) if i == 0 or layers[i] != layers[i - 1]]
        rows = []
        for i in range(c.k):
            first = max(j for j in firsts if j <= i)
            count = sum(1 for t in layers if t == layers[first])
            rows.append(len(self.fused) * first + f * count + (i - first))
        z = self.ht_get_buffer(HT_BUF_FUSED_DRAFT_LOGITS)
        return z[rows], self.ht_get_buffer(HT_BUF_FUSED_CANDIDATES)[f]

    def ht_cache_len(self) -> int:
        return lib.ht_cache_len(self.handle)

    def ht_get_buffer(self, which: int, layer: int = 0):
        """Device buffer as a torch tensor view (read-only by convention)."""
        torch = self.torch
        p, nb = C.c_void_p(), C.c_size_t()
        _check(lib.ht_get_buffer(self.handle, which, layer, C.byref(p), C.byref(nb)))
        off = p.value - self.workspace.data_ptr()
        raw = self.workspace[off:off + nb.value]
        c = self.cfg
        mdt = torch.float32 if c.dtype == HT_F32 else torch.bfloat16
        if which == HT_BUF_DRAFT_LOGITS:
            return raw.view(torch.float32).view(c.k, c.vocab)
        if which == HT_BUF_CANDIDATES:
            return raw.view(torch.int32).view(c.k, HT_MAX_TOPK)
        if which == HT_BUF_FUSED_DRAFT_LOGITS:
            return raw.view(torch.float32).view(-1, c.vocab)
        if which == HT_BUF_FUSED_CANDIDATES:
            return raw.view(torch.int32).view(-1, c.k, HT_MAX_TOPK)
        if which == HT_BUF_CANDIDATE_LOGPROBS:
            return raw.view(torch.float32).view(c.k, HT_MAX_TOPK)
        if which in (HT_BUF_TREE_TOKENS, HT_BUF_ROOT, HT_BUF_TREE_PARENT, HT_BUF_TREE_RANK):
            return raw.view(torch.int32)
        if which == HT_BUF_SAVED_HIDDEN:
            return raw.view(torch.float32).view(-1, c.d_model)
        if which == HT_BUF_TRANSFER_SRC:
            return raw.view(torch.float32)
        if which == HT_BUF_PSEUDO:
            return raw.view(torch.float32).view(c.k, c.d_model)
        if which == HT_BUF_K_CACHE:
            return raw.view(mdt).view(c.max_cache, c.n_kv_heads, c.head_dim)
        if which == HT_BUF_V_CACHE:
            return raw.view(mdt).view(c.n_kv_heads, c.head_dim, c.max_cache)
        raise ValueError(which)
