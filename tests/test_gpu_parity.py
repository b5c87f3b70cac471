"""Parity of the HIP path against the CPU oracle, through the C ABI.  Needs a real MI355X.

Tolerances: fp32 model logits max-abs <= 1e-4; bf16, per row: max-abs error <= 3e-2 * max|reference| and
relative L2 error <= 3e-2.
Integer stages (top-k, tree tokens, arg-max, acceptance path, accepted count) are compared bit-exactly
against the oracle's rules applied to the GPU's own logits, and on the fp32 model also against the
fp64 oracle's integers, with the smallest logit margin of the run asserted to be far above tolerance.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from ht_inputs import WORKLOADS, make_weights, counter_normal, random_tree, chain_tree, star_tree, prune_tree
from ht_inputs.workloads import ATTENTION_OP
from oracle import ht_oracle as O
from helpers import torch_dtype, oracle_model, prompt_of, tree_of, small_workload


def _B():
    import paper_2404_12022_amd.binding as B
    return B


def _H():
    import gpu_harness as H
    return H


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ inputs
def test_generators_give_the_same_bits_on_the_gpu():
    for dt in (torch.float32, torch.bfloat16):
        a = counter_normal(7, 1001, (300, 129), 0.02, device="cpu", dtype=dt)
        b = counter_normal(7, 1001, (300, 129), 0.02, device="cuda:0", dtype=dt)
        assert torch.equal(a, b.cpu())
    g = counter_normal(7, 2, (4096,), 0.02, mean=1.0, device="cuda:0")
    assert torch.equal(g.cpu(), counter_normal(7, 2, (4096,), 0.02, mean=1.0))


# ------------------------------------------------------------------ skinny product, op level
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (3, 208, 200), (8, 1024, 256), (16, 768, 688), (17, 4096, 1024),
                                   (64, 8192, 512), (64, 1024, 4096), (76, 2064, 688), (84, 4096, 1024), (96, 22016, 256),
                                   (100, 256, 11008), (128, 12288, 128),
                                   (40, 5120, 13824), (67, 5136, 12296),    # 128-row workgroups, six K splits
                                   (129, 1024, 4096), (200, 2064, 688), (256, 12288, 128), (144, 5120, 13824)])  # two launches
def test_skinny_product_matches_textbook_product(dtype, M, N, K):
    B, H = _B(), _H()
    say(f"gemm {dtype} M={M} N={N} K={K}")
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Mp = B.ht_padded_rows(M)
    a = torch.zeros(Mp, K, dtype=tdt, device=H.DEV)
    a[:M] = counter_normal(1, 11, (M, K), 1.0, device=H.DEV, dtype=tdt)
    w = counter_normal(1, 12, (N, K), 0.05, device=H.DEV, dtype=tdt)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device=H.DEV)
    scratch = torch.empty(B.ht_skinny_gemm_scratch_bytes(M, N, K), dtype=torch.uint8, device=H.DEV)
    B.ht_skinny_gemm(a, w, M, N, K, B.HT_F32 if dtype == "f32" else B.HT_BF16, out, scratch)
    torch.cuda.synchronize()
    want = O.linear(H.cpu(a[:M]), H.cpu(w))
    got = H.cpu(out)
    assert np.all(np.isfinite(got))
    # inputs are exact in both paths; only fp32 accumulation order differs
    bound = 2e-5 * np.sqrt(K) * np.abs(H.cpu(a[:M])).max() * 0.05 * 8 + 1e-6
    assert np.max(np.abs(got - want)) <= bound, (np.max(np.abs(got - want)), bound)


@pytest.mark.parametrize("M,f,K", [(1, 64, 64), (7, 208, 200), (64, 688, 256), (76, 1376, 512), (128, 4112, 136),
                                   (64, 11008, 128), (131, 688, 256), (256, 1376, 512)])
def test_fused_gate_up_product_matches_its_definition(M, f, K):
    """act = silu(a . Wg^T) * (a . Wu^T) (the feed-forward block's first half, fused into one kernel) against the
    oracle's product and SiLU, bf16 operands; sizes with ragged row-block counts and several token tiles."""
    B, H = _B(), _H()
    say(f"gate/up M={M} f={f} K={K}")
    Mp = B.ht_padded_rows(M)
    a = torch.zeros(Mp, K, dtype=torch.bfloat16, device=H.DEV)
    a[:M] = counter_normal(3, 31, (M, K), 1.0, device=H.DEV, dtype=torch.bfloat16)
    wg = counter_normal(3, 32, (f, K), 0.1, device=H.DEV, dtype=torch.bfloat16)
    wu = counter_normal(3, 33, (f, K), 0.1, device=H.DEV, dtype=torch.bfloat16)
    packed = torch.empty(B.ht_weight_pack_bytes(2 * f, K), dtype=torch.uint8, device=H.DEV)
    B.ht_gate_up_pack(wg, wu, f, K, packed)
    out = torch.full((M, f), float("nan"), dtype=torch.bfloat16, device=H.DEV)
    B.ht_gate_up_silu_packed(a, packed, M, f, K, out)
    torch.cuda.synchronize()
    x = H.cpu(a[:M])
    want = O.silu(O.linear(x, H.cpu(wg))) * O.linear(x, H.cpu(wu))
    got = H.cpu(out)
    assert np.all(np.isfinite(got))
    # fp32 sums of exact bf16 products, one bf16 rounding of the result (2^-9 relative)
    assert np.max(np.abs(got - want) - 2.0 ** -8 * np.abs(want)) <= 1e-5 * np.sqrt(K) * np.abs(want).max() + 1e-6
    with pytest.raises(B.HTError) as e:
        B.ht_gate_up_silu_packed(a, packed, M, f + 8, K, out)
    assert e.value.code == B.HT_EINVAL


def test_matrix_core_probe_counts_its_work_and_rejects_bad_arguments():
    B, H = _B(), _H()
    sink = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    # 512 workgroups x 4 wavefronts x iters x (32 instructions of 2 * 16 * 16 * 32 | 8 of 2 * 32 * 32 * 16) operations
    assert B.ht_mfma_rate_probe(0, 10, sink) == 512 * 4 * 10 * 32 * 16384
    assert B.ht_mfma_rate_probe(1, 10, sink) == 512 * 4 * 10 * 8 * 32768
    assert B.ht_mfma_rate_probe(2, 3, sink) == 512 * 4 * 3 * 32 * 16384           # the same with hashed operand bits
    assert B.ht_mfma_rate_probe(3, 3, sink) == 512 * 4 * 3 * 8 * 32768
    torch.cuda.synchronize()
    assert int(sink[0]) == 0
    for form, iters in ((4, 10), (-1, 10), (0, 0), (0, (1 << 20) + 1)):
        with pytest.raises(B.HTError) as e:
            B.ht_mfma_rate_probe(form, iters, sink)
        assert e.value.code == B.HT_EINVAL


def test_stream_read_probe_reads_whole_passes_and_rejects_bad_buffers():
    B, H = _B(), _H()
    buf = torch.zeros(40 << 20, dtype=torch.uint8, device=H.DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=H.DEV)
    assert B.ht_stream_read_probe(buf, sink) == 40 << 20            # 256 workgroups x 5 x 32 KiB
    assert B.ht_stream_read_probe(buf[:(20 << 20) + 4096], sink) == 16 << 20
    torch.cuda.synchronize()
    assert int(sink[0]) == 0
    for bad in (buf[:1 << 20], buf[8:(9 << 20)]):                   # under one pass; misaligned
        with pytest.raises(B.HTError) as e:
            B.ht_stream_read_probe(bad, sink)
        assert e.value.code == B.HT_EINVAL


# ------------------------------------------------------------------ tree attention, op level
def _attention_case(dtype, T, n, Hq, Hkv, hd, parent, seed, cap=None, rotate=True, base=10000.0, poison=False):
    """poison: the cache slots past the last tree row hold NaN (they are never visible and must not leak)."""
    B, H = _B(), _H()
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    cap = cap or ((n + T + 7) // 8 * 8 + (24 if poison else 0))
    q = counter_normal(seed, 21, (T, Hq, hd), 1.0, device=H.DEV, dtype=tdt)
    kc = counter_normal(seed, 22, (cap, Hkv, hd), 1.0, device=H.DEV, dtype=tdt)
    vc = counter_normal(seed, 23, (Hkv, hd, cap), 1.0, device=H.DEV, dtype=tdt)
    if poison:
        kc[n + T:] = float("nan")
        vc[:, :, n + T:] = float("nan")
    kn = counter_normal(seed, 24, (T, Hkv, hd), 1.0, device=H.DEV, dtype=tdt)
    vn = counter_normal(seed, 25, (T, Hkv, hd), 1.0, device=H.DEV, dtype=tdt)
    out = torch.full((T, Hq * hd), float("nan"), dtype=tdt, device=H.DEV)
    scratch = torch.empty(B.ht_tree_attention_scratch_bytes(T, Hq, hd), dtype=torch.uint8, device=H.DEV)
    depth = O.tree_depth(parent)
    pos = np.array([n + e for e in depth])
    k_old = H.cpu(kc)[:n]
    v_old = np.transpose(H.cpu(vc), (2, 0, 1))[:n]
    if rotate:
        B.ht_tree_attention(q, kn, vn, kc, vc, cap, n, T, parent, Hq, Hkv, hd, B.HT_F32 if dtype == "f32" else B.HT_BF16,
                            base, out, scratch)
        qq, kk, vv = O.rope(H.cpu(q), pos, base), O.rope(H.cpu(kn), pos, base), H.cpu(vn)
    else:
        kc[n:n + T] = kn
        vc[:, :, n:n + T] = vn.permute(1, 2, 0)
        B.ht_tree_attention(q, None, None, kc, vc, cap, n, T, parent, Hq, Hkv, hd,
                            B.HT_F32 if dtype == "f32" else B.HT_BF16, base, out, scratch)
        qq, kk, vv = H.cpu(q), H.cpu(kn), H.cpu(vn)
    torch.cuda.synchronize()
    if not rotate:                              # parent = None: the tables left in scratch serve the same tree again
        first = out.clone()
        out.fill_(float("nan"))
        B.ht_tree_attention(q, None, None, kc, vc, cap, n, T, None, Hq, Hkv, hd,
                            B.HT_F32 if dtype == "f32" else B.HT_BF16, base, out, scratch)
        torch.cuda.synchronize()
        assert torch.equal(first, out), "reusing the uploaded tree tables changed the result"
    vis = np.concatenate([np.ones((T, n), dtype=bool), O.ancestor_matrix(parent)], axis=1)
    want = O.masked_attention(qq, np.concatenate([k_old, kk]), np.concatenate([v_old, vv]), vis).reshape(T, Hq * hd)
    got = H.cpu(out)
    assert np.all(np.isfinite(got))
    if dtype == "f32":
        assert np.max(np.abs(got - want)) <= 2e-5, np.max(np.abs(got - want))
    else:
        # bf16: rotated q/k and the output are rounded to bf16 (2^-9 relative each); scores of size ~sqrt(hd)
        # move the softmax weights by up to ~2e-2, values are O(1)
        ok, worst = H.within_bf16(got, want, 3e-2)
        assert ok, worst
    if rotate:                                      # appended rows landed in slots n..n+T-1
        assert_k = H.cpu(kc)[n:n + T]
        if dtype == "f32":
            assert np.max(np.abs(assert_k - kk)) <= 1e-5
        else:
            assert H.within_bf16(assert_k, kk, 1e-2)[0]
        assert torch.equal(vc[:, :, n:n + T], vn.permute(1, 2, 0))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", ["random", "chain", "star", "single", "gqa", "empty_cache", "no_rotate", "ragged",
                                  "rows200", "rows256", "long_ragged", "long_grouped", "long_grouped_few_rows",
                                  "long_grouped_one_row"])
def test_tree_attention_small(dtype, case):
    say(f"attention {dtype} {case}")
    if case == "random":
        _attention_case(dtype, 24, 37, 4, 4, 64, random_tree(5, 24, 4)[0], 3)
    elif case == "chain":
        _attention_case(dtype, 9, 64, 2, 2, 128, chain_tree(9)[0], 4)
    elif case == "star":
        _attention_case(dtype, 17, 100, 2, 2, 128, star_tree(17)[0], 5)
    elif case == "single":
        _attention_case(dtype, 1, 33, 4, 4, 64, [-1], 6)
    elif case == "gqa":
        _attention_case(dtype, 20, 70, 8, 2, 128, random_tree(8, 20, 5)[0], 7)
    elif case == "empty_cache":
        _attention_case(dtype, 12, 0, 2, 2, 64, random_tree(9, 12, 3)[0], 8)
    elif case == "no_rotate":
        _attention_case(dtype, 24, 37, 4, 4, 64, random_tree(5, 24, 4)[0], 9, rotate=False)
    elif case == "ragged":
        _attention_case(dtype, 70, 203, 3, 3, 128, random_tree(11, 70, 6)[0], 10, poison=True)
    elif case == "long_ragged":                      # 33 tiles, the last one holding two keys and then NaN
        _attention_case(dtype, 50, 2000, 4, 2, 128, random_tree(14, 50, 5)[0], 13, poison=True)
    elif case == "long_grouped_few_rows":            # under 17 rows with four query heads per key/value head
        _attention_case(dtype, 5, 1900, 8, 2, 128, random_tree(16, 5, 3)[0], 15, poison=True)
    elif case == "long_grouped_one_row":
        _attention_case(dtype, 1, 4099, 16, 2, 64, [-1], 16, poison=True)
    elif case == "long_grouped":                     # six query heads on one key/value head, 64-wide heads, ragged end
        _attention_case(dtype, 40, 1777, 6, 1, 64, random_tree(15, 40, 4)[0], 14, poison=True)
    elif case == "rows200":                          # more rows than a tree has nodes: four ancestor-mask words
        _attention_case(dtype, 200, 150, 2, 1, 128, random_tree(12, 200, 9)[0], 11)
    else:
        _attention_case(dtype, 256, 61, 2, 2, 64, random_tree(13, 256, 12)[0], 12, rotate=False)


def test_tree_attention_at_the_op_workload_size():
    a = ATTENTION_OP
    say("attention bf16 op workload")
    parent, _ = random_tree(a["seed"], a["tree_size"], a["max_depth"])
    _attention_case("bf16", a["tree_size"], a["cache_len"], a["n_heads"], a["n_kv_heads"], a["head_dim"], parent,
                    a["seed"], cap=a["cache_len"] + a["tree_size"], base=a["rope_base"])


def test_tree_attention_grouped_queries_over_a_long_cache():
    """The 70B-shaped attention: 64 query heads on 8 key/value heads, 4096 cached keys, a 64-node tree."""
    say("attention bf16 Hq 64 / Hkv 8, n = 4096, T = 64")
    _attention_case("bf16", 64, 4096, 64, 8, 128, random_tree(70, 64, 4)[0], 70, cap=4160)


# ------------------------------------------------------------------ end to end, tiny model
@pytest.mark.parametrize("name", ["tiny", "tiny_k3", "tiny_full7", "tiny_t123", "tiny_t112"])
def test_tiny_fp32_sixteen_steps_match_oracle_and_greedy(name):
    H = _H()
    wl = WORKLOADS[name]
    say(f"end-to-end {name}")
    sc = H.StepCompare(wl)
    sc.check_prefill()
    out = []
    for step in range(16):
        out += sc.step()["emitted"]
    want = sc.model.ar_greedy(sc.prompt, len(out))
    assert out == want                                               # losslessness on the GPU
    sc.check_cache("after 16 steps")
    # no near-tie could hide or fake a mismatch: every decision of the run (top-1/top-2 of each verify row,
    # neighbouring draft candidates) has a margin above the tolerance and 10x above the error actually seen
    say(f"{name}: smallest decision margin {sc.min_margin:.3e}, largest logit error {sc.max_err:.3e}")
    assert sc.min_margin > H.FP32_LOGIT_TOL and sc.min_margin > 10 * sc.max_err, (sc.min_margin, sc.max_err)


@pytest.mark.parametrize("name,side_stream", [("tiny", False), ("tiny_t123", False), ("tiny", True)])
def test_tiny_fp32_decode_reproduces_the_stored_trace(name, side_stream):
    """The same decode as the trace under tests/golden/ (written from the oracle alone), through the C ABI only:
    tree tokens, accepted path, emitted tokens, pending root and cache length of all 16 steps."""
    from test_golden import read_trace
    B, H = _B(), _H()
    want = read_trace()[name]
    wl = WORKLOADS[name]
    say(f"stored trace {name}")
    parent, rank = tree_of(wl)
    gpu = H.gpu_model(wl, max_tree=len(parent))
    torch.cuda.synchronize()
    # every call takes the stream it is to run on; with side_stream all of them go to one that is not the default
    stream = torch.cuda.Stream() if side_stream else torch.cuda.current_stream()
    with torch.cuda.stream(stream):
        gpu.ht_set_tree(parent, rank, stream)
        gpu.ht_prefill(prompt_of(wl), stream)
        stream.synchronize()
        assert int(gpu.ht_get_buffer(B.HT_BUF_ROOT)[0].item()) == want["root"]
        for s, st in enumerate(want["steps"]):
            gpu.ht_transfer(None, None, stream)
            gpu.ht_tree_verify_step(None, None, None, stream)
            stream.synchronize()
            tok = [int(t) for t in gpu.ht_get_buffer(B.HT_BUF_TREE_TOKENS).cpu()]
            assert tok == st["tok"], f"step {s}: tree tokens"
            m, emitted, root, path = gpu.ht_accept_and_compact(stream)
            assert (m, path, emitted) == (len(st["path"]), st["path"], st["emitted"]), f"step {s}: acceptance"
            assert (root, gpu.ht_cache_len()) == (st["next_root"], st["cache_len"]), f"step {s}: state"
    gpu.close()


@pytest.mark.parametrize("fused", [False, True])
def test_decode_loop_gives_the_greedy_continuation_until_the_cache_is_full(fused):
    """`HTModel.decode` (the ABI calls in a loop) on the tiny workload: the text is the oracle's greedy
    autoregressive continuation (Sec. 4.1: verification keeps the output of plain greedy decoding), with and
    without pseudo rows riding in the verify pass, and the loop stops before a pass would overflow the cache."""
    B, H = _B(), _H()
    wl = WORKLOADS["tiny"].with_(max_cache=80)
    parent, rank = tree_of(wl)
    nodes = _rank0_chain(parent, rank) if fused else []
    say(f"decode loop, fused nodes {nodes}")
    gpu = H.gpu_model(wl, max_tree=len(parent) + len(nodes) * wl.k)
    gpu.ht_set_tree(parent, rank)
    if nodes:
        gpu.ht_set_fused_nodes(nodes)
    prompt = prompt_of(wl)
    gpu.ht_prefill(prompt)
    out = gpu.decode(20)
    assert len(out) >= 20
    assert out == oracle_model(wl).ar_greedy(prompt, len(out))
    more = gpu.decode(10 ** 6)                               # runs into the capacity check, never past it
    rows = len(parent) + len(nodes) * wl.k
    assert gpu.ht_cache_len() + rows > wl.max_cache >= gpu.ht_cache_len()
    assert out + more == oracle_model(wl).ar_greedy(prompt, len(out) + len(more))
    gpu.close()


@pytest.mark.parametrize("name", ["tiny", "tiny_t123"])
def test_device_resident_loop_reproduces_the_stored_trace(name):
    """`ht_decode_steps`: 16 steps with the cache length kept on the device and one host wait at the end give the
    tokens, counts and final state of the stored trace (16 single steps of the oracle); the state it leaves is a
    valid starting point for ordinary single steps, checked against the oracle."""
    from test_golden import read_trace
    B, H = _B(), _H()
    want = read_trace()[name]
    wl = WORKLOADS[name]
    say(f"device-resident loop {name}")
    sc = H.StepCompare(wl)
    for part in ((0, 5), (5, 16)):                                # two calls: the second starts from the first's state
        counts, toks, root = sc.gpu.ht_decode_steps(part[1] - part[0])
        steps = want["steps"][part[0]:part[1]]
        assert counts == [len(st["path"]) for st in steps]
        assert toks == [t for st in steps for t in st["emitted"]]
        assert (root, sc.gpu.ht_cache_len()) == (steps[-1]["next_root"], steps[-1]["cache_len"])
    for _ in range(16):                                           # bring the oracle to the same point
        sc.ora.step()
    assert int(sc.gpu.ht_get_buffer(B.HT_BUF_ROOT)[0].item()) == sc.ora.root
    sc.check_cache("after the loop")
    for _ in range(3):                                            # single steps go on from the loop's state
        sc.step()
    with pytest.raises(B.HTError) as e:
        sc.gpu.ht_decode_steps(0)
    assert e.value.code == B.HT_EINVAL
    with pytest.raises(B.HTError) as e:
        sc.gpu.ht_decode_steps(64)                                # 64 steps of up to k + 1 tokens do not fit the cache
    assert e.value.code == B.HT_ECAPACITY
    sc.gpu.close()


def test_device_resident_loop_sixty_four_steps_give_greedy_text():
    """The most steps one call takes, on the tiny model: the text is the greedy continuation, the counts add up."""
    B, H = _B(), _H()
    wl = WORKLOADS["tiny"].with_(max_cache=256)
    parent, rank = tree_of(wl)
    gpu = H.gpu_model(wl, max_tree=len(parent))
    gpu.ht_set_tree(parent, rank)
    prompt = prompt_of(wl)
    gpu.ht_prefill(prompt)
    counts, toks, root = gpu.ht_decode_steps(B.HT_MAX_LOOP_STEPS)
    assert len(counts) == 64 and all(1 <= c <= wl.k + 1 for c in counts) and sum(counts) == len(toks)
    want = oracle_model(wl).ar_greedy(prompt, len(toks) + 1)
    assert toks == want[:-1] and root == want[-1]
    assert gpu.ht_cache_len() == len(prompt) + len(toks)
    say(f"64 steps in one call: {len(toks)} tokens, {max(counts)} at most per step")
    gpu.close()


def test_device_resident_loop_on_the_matrix_core_path():
    """The loop against single steps of the same library on a 7B-wide bf16 model (2 layers): both run the same
    kernels on the same values, so tokens, counts and the caches agree bit for bit."""
    B, H = _B(), _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), prompt_len=100, max_cache=256)
    parent, rank = tree_of(wl)
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    say("device-resident loop, 7B width")
    a, b = H.gpu_model(wl, tensors, max_tree=len(parent)), H.gpu_model(wl, tensors, max_tree=len(parent))
    for g in (a, b):
        g.ht_set_tree(parent, rank)
        g.ht_prefill(prompt_of(wl))
    steps = 6
    counts, toks, root = a.ht_decode_steps(steps)
    ref_counts, ref_toks = [], []
    for _ in range(steps):
        b.ht_transfer(None, None)
        b.ht_tree_verify_step(None, None, None)
        m, emitted, ref_root, _ = b.ht_accept_and_compact()
        ref_counts.append(m)
        ref_toks += emitted
    assert (counts, toks, root) == (ref_counts, ref_toks, ref_root)
    assert a.ht_cache_len() == b.ht_cache_len() == wl.prompt_len + sum(counts)
    n = a.ht_cache_len()
    for layer in (0, 1):
        assert torch.equal(a.ht_get_buffer(B.HT_BUF_K_CACHE, layer)[:n], b.ht_get_buffer(B.HT_BUF_K_CACHE, layer)[:n])
        assert torch.equal(a.ht_get_buffer(B.HT_BUF_V_CACHE, layer)[:, :, :n], b.ht_get_buffer(B.HT_BUF_V_CACHE, layer)[:, :, :n])
    a.close()
    b.close()


def _rank0_chain(parent, rank):
    chain, cur = [0], 0
    while True:
        kids = [v for v in range(len(parent)) if parent[v] == cur and rank[v] == 0]
        if not kids:
            return chain
        cur = kids[0]
        chain.append(cur)


@pytest.mark.parametrize("name,which", [("tiny", "all"), ("tiny_k3", "all"), ("tiny_full7", "all"), ("tiny", "root"),
                                        ("tiny_k3", "chain"), ("tiny_t123", "all"), ("tiny_t112", "chain")])
def test_tiny_fp32_drafting_inside_the_verify_pass(name, which):
    """Pseudo rows of chosen tree nodes ride along in the verify pass (Fig. 2 caption, end of Sec. 3.4).  The draft
    distributions they give must equal the oracle's, which drafts after acceptance, and the decoded text must
    still be the greedy one; nodes outside the chosen set fall back to drafting after acceptance."""
    H = _H()
    wl = WORKLOADS[name]
    parent, rank = tree_of(wl)
    fused = {"all": list(range(len(parent))), "root": [0], "chain": _rank0_chain(parent, rank)}[which]
    say(f"in-pass drafting {name}, nodes {fused}")
    sc = H.StepCompare(wl, fused=fused)
    out = []
    for step in range(16):
        out += sc.step()["emitted"]
    assert out == sc.model.ar_greedy(sc.prompt, len(out))
    sc.check_cache("after 16 steps")
    say(f"{name}/{which}: {sc.steps_without_draft_pass} of 16 steps needed no draft pass, smallest margin "
        f"{sc.min_margin:.3e}, largest logit error {sc.max_err:.3e}")
    assert sc.steps_without_draft_pass >= (15 if which == "all" else 1)
    assert sc.min_margin > H.FP32_LOGIT_TOL and sc.min_margin > 10 * sc.max_err, (sc.min_margin, sc.max_err)
    sc.gpu.close()


def _full_fused_schedule_case(wl, tensors_gpu, tensors_cpu, prompt_len):
    """The paper's own inference schedule (Fig. 2 caption, end of Sec. 3.4): EVERY tree node carries its k pseudo rows
    through the verify pass, T (1 + k) rows in the blocks above the transfer layer.  One pass on given tokens against
    the oracle's `fused_verify_and_draft`: the T verify-logit rows, and the k draft distributions of every node."""
    B, H = _B(), _H()
    parent, rank = tree_of(wl)
    T = len(parent)
    model = oracle_model(wl, tensors_cpu)
    ora = O.HiddenTransferOracle(model, parent, rank, wl.max_cache)
    prompt = prompt_of(wl, prompt_len)
    ora.prefill(prompt)
    gpu = H.gpu_model(wl, tensors_gpu, max_tree=T * (1 + wl.k))
    gpu.ht_set_tree(parent, rank)
    gpu.ht_set_fused_nodes(list(range(T)))
    gpu.ht_prefill(prompt)
    tok = [ora.root] + [(11 + 17 * v) % wl.vocab for v in range(1, T)]
    z_o, g_o, d_o = ora.fused_verify_and_draft(tok)
    z = torch.empty(T, wl.vocab, dtype=torch.float32, device=H.DEV)
    g = torch.empty(T, dtype=torch.int32, device=H.DEV)
    gpu.ht_tree_verify_step(torch.tensor(tok, dtype=torch.int32, device=H.DEV), g, z)
    torch.cuda.synchronize()
    worst = H.assert_close(H.cpu(z), z_o, wl.dtype, "verify logits with every node drafting in the pass")
    zc = H.cpu(z)
    assert [int(t) for t in g.cpu()] == [int(j) for j in np.argmax(zc, axis=1)]
    width, cands = ora.width, []
    for v in range(T):
        d, cand = gpu.fused_drafts(v)
        d = H.cpu(d)
        worst = max(worst, H.assert_close(d, d_o[v], wl.dtype, f"draft distributions of node {v}"))
        cands.append(cand.cpu().numpy())
        for e in range(1, len(width)):          # the oracle's candidate rule on the GPU's own draft logits
            assert list(cands[v][e - 1][:width[e]]) == O.top_candidates(d[e - 1], width[e]), f"node {v}: candidates at depth {e}"
    # the step after any acceptance needs neither a transfer nor a draft pass: its tree comes from these rows
    m, emitted, root, path = gpu.ht_accept_and_compact()
    gpu.ht_transfer(None, None)
    gpu.ht_tree_verify_step(None, g, z)
    torch.cuda.synchronize()
    tok2 = [int(t) for t in gpu.ht_get_buffer(B.HT_BUF_TREE_TOKENS).cpu()]
    mine = cands[path[-1]]
    assert tok2 == [root] + [int(mine[ora.depth[v] - 1][ora.rank[v]]) for v in range(1, T)], "tree of the next step"
    gpu.close()
    return worst


@pytest.mark.parametrize("name", ["tiny", "tiny_k3", "tiny_t123"])
def test_every_node_drafts_inside_the_verify_pass_tiny(name):
    wl = WORKLOADS[name]
    say(f"full fused schedule {name}: {wl.tree_size} nodes x (1 + {wl.k}) rows")
    worst = _full_fused_schedule_case(wl, None, None, wl.prompt_len)
    say(f"  largest logit error {worst:.3e}")


def test_every_node_drafts_inside_the_verify_pass_llama7b_width():
    """64 nodes x (1 + 3) = 256 rows in the upper block and the LM head at the 7B widths (2 layers, transfer after the
    first): the projections run two launches of 128 rows over the same weights, attention four row groups."""
    H = _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), prompt_len=96, max_cache=96 + 256 + 16)
    say("full fused schedule, 7B width, 2 layers: 256 rows above the transfer layer")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    worst = _full_fused_schedule_case(wl, tensors, cpu_tensors, wl.prompt_len)
    say(f"  worst logit error / bound {worst:.3f}")


@pytest.mark.parametrize("seed", range(6))
def test_random_trees_with_random_drafting_nodes(seed):
    """Irregular trees (random attachment, depth up to k) with a random subset of nodes drafting inside the verify
    pass, on the model with a transfer layer per step: tables, joins and candidate maps for arbitrary shapes."""
    H = _H()
    wl = WORKLOADS["tiny_t123"]
    T = 5 + 2 * seed
    parent, rank = random_tree(100 + seed, T, wl.k)
    pick = np.random.default_rng(seed).permutation(T)[: 1 + seed % 4]
    fused = sorted(int(v) for v in pick)
    say(f"random tree seed {seed}: T={T} parent={parent} drafting nodes {fused}")
    sc = H.StepCompare(wl, tree=(parent, rank), fused=fused)
    out = []
    for step in range(8):
        out += sc.step()["emitted"]
    assert out == sc.model.ar_greedy(sc.prompt, len(out))
    sc.check_cache("after 8 steps")
    sc.gpu.close()


def _random_shape(seed):
    """A small model with dimensions drawn at random from what the configuration check allows: odd head counts and
    group sizes, head sizes with and without a matrix-core attention kernel, widths that do and do not fit the
    packed weight layout, 1..4 transfer steps at non-decreasing random layers, a random tree with random drafting
    nodes, a prompt that is not a multiple of anything."""
    rng = np.random.default_rng(4000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    hd = int(rng.choice([16, 32, 64, 128] if dtype == "bf16" else [8, 16, 32, 64]))
    hkv = int(rng.choice([1, 2, 3]))
    hq = hkv * int(rng.choice([1, 2, 4]))
    d = int(rng.choice([64, 96, 136, 160, 256]))
    f = int(rng.choice([72, 128, 200, 344]))
    vocab = int(rng.choice([128, 250, 512, 1000]))
    layers = int(rng.integers(2, 5))
    k = int(rng.integers(1, 5))
    t = tuple(sorted(int(x) for x in rng.integers(1, layers, size=k)))
    T = int(rng.integers(2, 41))
    parent, rank = random_tree(4000 + seed, T, k)
    n_fused = int(rng.integers(0, min(T, (128 - T) // k) + 1))
    fused = sorted(int(v) for v in rng.permutation(T)[:min(n_fused, 6)])
    prompt_len = int(rng.integers(3, 71))
    rows = T + len(fused) * k
    max_cache = (prompt_len + 5 * (k + 1) + rows + 7) // 8 * 8
    branching = tuple(1 + max(rank[v] for v in range(T) if len(_path_to(parent, v)) - 1 == e) for e in range(1, k + 1)
                      if any(len(_path_to(parent, v)) - 1 == e for v in range(T)))
    wl = small_workload(name=f"fuzz{seed}", n_layers=layers, d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=hd, d_ffn=f,
                        vocab=vocab, k=k, transfer_layers=t, dtype=dtype, prompt_len=prompt_len, max_cache=max_cache,
                        tree_size=T, branching=branching, seed=7000 + seed)
    return wl, (parent, rank), fused


def _path_to(parent, v):
    p = []
    while v >= 0:
        p.append(v)
        v = parent[v]
    return p


def _random_packed_shape(seed):
    """Random bf16 shapes that all run on the matrix-core kernels (packed projections, fused q|k|v epilogue or its
    split fallback, both attention kernels): widths in multiples of 16, heads of 64 or 128, up to 128 rows a pass."""
    rng = np.random.default_rng(5000 + seed)
    hd = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 5]))
    hq = hkv * int(rng.choice([1, 2, 4]))
    d = 16 * int(rng.integers(8, 49))
    f = 16 * int(rng.integers(6, 90))
    vocab = 16 * int(rng.integers(20, 130))
    layers = int(rng.integers(2, 4))
    k = int(rng.integers(1, 6))
    t = tuple(sorted(int(x) for x in rng.integers(1, layers, size=k)))
    T = min(int(rng.choice([1, 3, 16, 17, 33, 64, 65, 90, 120])), 1 + 40 * k)     # a parent offers at most 64 candidates
    parent, rank = random_tree(5000 + seed, T, k) if T > 1 else ([-1], [0])
    room = (128 - T) // k
    fused = sorted(int(v) for v in rng.permutation(T)[:int(rng.integers(0, min(T, room) + 1))])
    prompt_len = int(rng.integers(1, 200))
    rows = max(T + len(fused) * k, k)
    max_cache = (prompt_len + 4 * (k + 1) + rows + 7) // 8 * 8
    wl = small_workload(name=f"packed{seed}", n_layers=layers, d_model=d, n_heads=hq, n_kv_heads=hkv, head_dim=hd, d_ffn=f,
                        vocab=vocab, k=k, transfer_layers=t, dtype="bf16", prompt_len=prompt_len, max_cache=max_cache,
                        tree_size=T, branching=(1,) * k, seed=8000 + seed)
    return wl, (parent, rank), fused


@pytest.mark.parametrize("seed", [f"any{i}" for i in range(12)] + [f"packed{i}" for i in range(12)])
def test_random_model_shapes_against_oracle(seed):
    H = _H()
    wl, tree, fused = _random_shape(int(seed[3:])) if seed.startswith("any") else _random_packed_shape(int(seed[6:]))
    say(f"random shape {seed}: {wl.dtype} layers={wl.n_layers} d={wl.d_model} heads={wl.n_heads}/{wl.n_kv_heads}x{wl.head_dim} "
        f"ffn={wl.d_ffn} vocab={wl.vocab} k={wl.k} t={wl.transfer_layers} T={wl.tree_size} drafting nodes {fused} "
        f"prompt {wl.prompt_len} cache {wl.max_cache}")
    sc = H.StepCompare(wl, tree=tree, fused=fused)
    sc.check_prefill()
    full = 0
    for step in range(4):
        r = sc.step(require_same_tokens=False)
        if r["emitted"] != r["oracle"]["emitted"] or r["root"] != r["oracle"]["root"]:
            break                       # a near-tie took the two decodes apart: what follows is not comparable
        full += 1
    say(f"  steps compared in full: {full}")
    if full == 4:
        sc.check_cache("after 4 steps")
    sc.gpu.close()
    if wl.dtype == "f32":
        assert full >= 1
    else:
        # bf16 decisions may part at a near-tie before a verify pass was compared: one more pass on given tokens,
        # which compares all T logit rows whatever was drafted
        sc = H.StepCompare(wl, tree=tree, fused=fused)
        sc.step(forced=[(7 + 13 * v) % wl.vocab for v in range(wl.tree_size)], require_same_tokens=False)
        sc.gpu.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_most_transfer_steps_the_interface_allows(dtype):
    """k = 8 transfer steps (the interface's maximum) at four distinct layers, a tree of depth 8, drafting nodes at
    several depths: eight pseudo rows per node join the passes in four groups."""
    H = _H()
    k = 8
    parent, rank = random_tree(77, 30, k)
    wl = small_workload(name="k8", n_layers=5, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=256, vocab=512,
                        k=k, transfer_layers=(1, 1, 2, 2, 3, 3, 4, 4), dtype=dtype, prompt_len=37, max_cache=200,
                        tree_size=30, branching=(1,) * k, seed=4242)
    fused = [0, 3, 9, 17]
    say(f"k = 8, {dtype}: tree depth {max(len(_path_to(parent, v)) for v in range(30)) - 1}, drafting nodes {fused}")
    sc = H.StepCompare(wl, tree=(parent, rank), fused=fused)
    sc.check_prefill()
    for step in range(4):
        r = sc.step(require_same_tokens=(dtype == "f32"))
        if r["emitted"] != r["oracle"]["emitted"] or r["root"] != r["oracle"]["root"]:
            break
    sc.gpu.close()


def test_long_cache_end_to_end_with_sixteen_key_slices():
    """A 6000-token prompt (47 prefill chunks) on a small packed bf16 model, then decode steps whose attention runs
    over 95 key tiles in sixteen slices, the most the merge handles; the one-token pass takes its own kernel."""
    H = _H()
    wl = small_workload(name="long", n_layers=2, d_model=128, n_heads=2, n_kv_heads=1, head_dim=64, d_ffn=256,
                        vocab=512, k=2, transfer_layers=(1, 1), dtype="bf16", prompt_len=6000, max_cache=6200,
                        tree_size=64, branching=(10, 6), seed=777)
    say("long cache: oracle prefill of 6000 tokens")
    sc = H.StepCompare(wl)
    sc.check_prefill()
    for step in range(2):
        r = sc.step(require_same_tokens=False)
        if r["emitted"] != r["oracle"]["emitted"] or r["root"] != r["oracle"]["root"]:
            break
    sc.gpu.close()
    sc = H.StepCompare(wl, tree=([-1], [0]))                       # the plain decode step at the same length
    sc.step(forced=[sc.ora.root], require_same_tokens=False)
    sc.gpu.close()


@pytest.mark.parametrize("name,fused", [("tiny_bf16", False), ("tiny_t123_bf16", False), ("tiny_t123_bf16", True)])
def test_tiny_bf16_sixteen_steps(name, fused):
    H = _H()
    wl = WORKLOADS[name]
    say(f"end-to-end {name}" + (" with in-pass drafts" if fused else ""))
    sc = H.StepCompare(wl, fused=_rank0_chain(*tree_of(wl)) if fused else None)
    sc.check_prefill()
    same = 0
    for step in range(16):
        r = sc.step(require_same_tokens=False)
        same += r["emitted"] == r["oracle"]["emitted"]
        if r["emitted"] != r["oracle"]["emitted"] or r["root"] != r["oracle"]["root"]:
            break                                                   # sequences diverged at a near-tie: stop comparing
    say(f"{name}: {same} steps with the oracle's tokens, {sc.verify_passes_compared} verify passes compared "
        f"({sc.steps_on_gpu_tree} on the GPU's own tree), worst logit error / bound {sc.max_err:.3f}")
    assert same >= 4 and sc.verify_passes_compared >= same
    sc.gpu.close()


@pytest.mark.parametrize("name", ["tiny", "tiny_k3", "tiny_bf16", "tiny_t123"])
def test_forced_acceptance_every_root_path(name):
    H = _H()
    wl = WORKLOADS[name]
    say(f"forced acceptance {name}")
    model = oracle_model(wl)
    prompt = prompt_of(wl, 10)
    truth = model.ar_greedy(prompt, wl.k + 3)
    parent, rank = tree_of(wl)
    tensors = make_weights(wl, wl.seed, H.DEV, torch_dtype(wl))
    seen = set()
    for leaf in range(len(parent)):
        full = []
        v = leaf
        while v >= 0:
            full.append(v)
            v = parent[v]
        full = full[::-1]
        for m_star in range(1, len(full) + 1):
            target = tuple(full[:m_star])
            if target in seen:
                continue
            seen.add(target)
            # odd cases also carry pseudo rows for the rank-0 chain: some forced paths end on it, some beside it
            fused = _rank0_chain(parent, rank) if len(seen) % 2 else None
            sc = H.StepCompare(wl, tensors_gpu=tensors, prompt=prompt, fused=fused)
            wrong = [t for t in range(wl.vocab) if t not in set(truth)]
            tok = [wrong[v] for v in range(len(parent))]
            for j, node in enumerate(target):
                tok[node] = truth[j]
            strict = wl.dtype == "f32"
            r = sc.step(forced=tok, require_same_tokens=strict)
            if strict:
                assert r["path"] == list(target) and r["emitted"] == truth[:m_star] and r["root"] == truth[m_star]
                nxt = sc.step()
                assert nxt["emitted"][0] == truth[m_star]
                sc.check_cache(f"after forced path {target}")
            sc.gpu.close()


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16"])
def test_exactly_tied_logits_resolve_to_lowest_ids(name):
    """LM head with only 64 distinct rows tiled over the vocabulary: every logit value occurs 16 times, so every
    arg-max and every top-k decision is a tie that must resolve by token id."""
    H = _H()
    wl = WORKLOADS[name]
    say(f"tied logits {name}")
    tensors = make_weights(wl, wl.seed, H.DEV, torch_dtype(wl))
    tensors["lm_head"] = tensors["lm_head"][:64].repeat(wl.vocab // 64, 1).contiguous()
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    sc = H.StepCompare(wl, tensors_gpu=tensors, tensors_cpu=cpu_tensors)
    for _ in range(4):
        r = sc.step(require_same_tokens=(wl.dtype == "f32"))
        assert all(t < 64 for t in r["emitted"]) and r["root"] < 64          # lowest id of each tie class
        cand = sc.gpu.ht_get_buffer(_B().HT_BUF_CANDIDATES).cpu().numpy()
        assert cand[0][1] == cand[0][0] + 64                                  # second best = same value, next id


def test_one_token_tree_is_a_plain_decode_step():
    H = _H()
    wl = WORKLOADS["tiny"]
    say("T=1 decode")
    sc = H.StepCompare(wl, tree=([-1], [0]))
    out = []
    for _ in range(8):
        out += sc.step()["emitted"]
    assert out == sc.model.ar_greedy(sc.prompt, 8)


def test_long_prompt_prefills_in_chunks():
    H = _H()
    wl = WORKLOADS["tiny"].with_(prompt_len=100)
    say("chunked prefill")
    sc = H.StepCompare(wl)
    sc.check_prefill()
    sc.step()


def test_deferred_layer_loading_gives_identical_results():
    """Projections supplied one layer at a time after ht_init_model (models larger than half the GPU memory)."""
    B, H = _B(), _H()
    wl = WORKLOADS["tiny_bf16"]
    say("deferred loading")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    parent, rank = tree_of(wl)
    prompt = prompt_of(wl)
    ref = B.HTModel(B.make_config(wl), tensors, H.DEV)
    lazy_tensors = dict(tensors)
    for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        lazy_tensors[name] = [None] * wl.n_layers
    lazy_tensors["lm_head"] = None
    lazy = B.HTModel(B.make_config(wl), lazy_tensors, H.DEV)
    lazy.ht_set_tree(parent, rank)
    with pytest.raises(B.HTError) as e:
        lazy.ht_prefill(prompt)
    assert e.value.code == B.HT_ESTATE
    for layer in reversed(range(wl.n_layers)):
        lazy.ht_load_layer(layer, {k: v[layer] for k, v in tensors.items() if isinstance(v, list) and k != "w_transfer"})
    lazy.ht_load_lm_head(tensors["lm_head"])
    outs = []
    for model in (ref, lazy):
        model.ht_set_tree(parent, rank)
        model.ht_prefill(prompt)
        z = torch.empty(len(parent), wl.vocab, dtype=torch.float32, device=H.DEV)
        model.ht_transfer()
        model.ht_tree_verify_step(None, None, z)
        outs.append((z.clone(), model.ht_accept_and_compact()))
    assert torch.equal(outs[0][0], outs[1][0]) and outs[0][1] == outs[1][1]
    f32 = WORKLOADS["tiny"]
    t32 = make_weights(f32, f32.seed, H.DEV, torch.float32)
    t32["lm_head"] = None
    with pytest.raises(B.HTError) as e:
        B.HTModel(B.make_config(f32), t32, H.DEV)                   # fp32 models cannot defer
    assert e.value.code == B.HT_EINVAL
    ref.close()
    lazy.close()


# ------------------------------------------------------------------ error paths (host-side validation)
def test_error_codes():
    B, H = _B(), _H()
    wl = WORKLOADS["tiny"]
    gpu = H.gpu_model(wl)
    parent, rank = tree_of(wl)
    with pytest.raises(B.HTError) as e:
        gpu.ht_tree_verify_step()
    assert e.value.code == B.HT_ESTATE
    for bad_parent in ([0] + parent[1:], parent[:3] + [5] + parent[4:]):
        with pytest.raises(B.HTError) as e:
            gpu.ht_set_tree(bad_parent, rank)
        assert e.value.code == B.HT_ETREE
    with pytest.raises(B.HTError) as e:
        gpu.ht_set_tree([-1, 0, 1, 2], [0, 0, 0, 0])                # depth 3 > k = 2
    assert e.value.code == B.HT_ETREE
    with pytest.raises(B.HTError) as e:
        gpu.ht_set_tree([-1, 0, 0], [0, 1, 1])                      # siblings share a rank
    assert e.value.code == B.HT_ETREE
    with pytest.raises(B.HTError) as e:
        gpu.ht_set_fused_nodes([0])                                 # no valid tree yet
    assert e.value.code == B.HT_ESTATE
    with pytest.raises(B.HTError) as e:
        H.gpu_model(WORKLOADS["tiny_t123"].with_(transfer_layers=(2, 1, 3)))   # transfer layers must not decrease
    assert e.value.code == B.HT_EINVAL
    gpu.ht_set_tree(parent, rank)
    with pytest.raises(B.HTError) as e:
        gpu.ht_set_fused_nodes([0])                                 # 8 + 2 rows > max_tree = 8
    assert e.value.code == B.HT_ECAPACITY
    with pytest.raises(B.HTError) as e:
        gpu.ht_tree_verify_step()
    assert e.value.code == B.HT_ESTATE                              # no prefill yet
    with pytest.raises(B.HTError) as e:
        gpu.ht_prefill([1, 2, wl.vocab])
    assert e.value.code == B.HT_EINVAL
    with pytest.raises(B.HTError) as e:
        gpu.ht_prefill(list(range(wl.max_cache + 1)))
    assert e.value.code == B.HT_ECAPACITY
    gpu.ht_prefill(prompt_of(wl, wl.max_cache - 4))
    with pytest.raises(B.HTError) as e:
        gpu.ht_tree_verify_step()                                   # drafting without ht_transfer
    assert e.value.code == B.HT_ESTATE
    gpu.ht_transfer()
    with pytest.raises(B.HTError) as e:
        gpu.ht_tree_verify_step()                                   # 124 + 8 > 128
    assert e.value.code == B.HT_ECAPACITY
    with pytest.raises(B.HTError) as e:
        gpu.ht_accept_and_compact()
    assert e.value.code == B.HT_ESTATE
    gpu.close()


# ------------------------------------------------------------------ large shapes
def _shallow_case(name, prompt_len, tree_size=None, cache=None, fused_chain=False, steps=1, layers=2, transfer_layers=None):
    """Full widths of a named workload (the launch configurations the benchmark uses), depth cut to 2 layers (or
    `layers`) and the prompt shortened so that the fp64 oracle finishes in seconds."""
    H = _H()
    base = WORKLOADS[name]
    T = tree_size or base.tree_size
    wl = base.with_(n_layers=layers, transfer_layers=transfer_layers or tuple(1 for _ in range(base.k)), prompt_len=prompt_len,
                    max_cache=cache or (prompt_len + 2 * T + 8 + 8 * steps) // 8 * 8, tree_size=T)
    say(f"{name} width, {layers} layers, T={T}, n={prompt_len}: generating weights")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    say(f"{name}: oracle + gpu")
    fused = _rank0_chain(*tree_of(wl)) if fused_chain else None
    sc = H.StepCompare(wl, tensors_gpu=tensors, tensors_cpu=cpu_tensors, fused=fused)
    sc.check_prefill()
    for step in range(steps):
        r = sc.step(require_same_tokens=False)
        say(f"{name}: emitted {r['emitted']} oracle {r['oracle']['emitted']} worst logit error / bound {sc.max_err:.3f}")
        if r["emitted"] != r["oracle"]["emitted"] or r["root"] != r["oracle"]["root"]:
            break                                       # a bf16 near-tie sent the two sequences apart: stop comparing
    else:
        sc.check_cache("after the steps")
    say(f"{name}: verify passes with all {T} logit rows held against the oracle: {sc.verify_passes_compared} "
        f"({sc.steps_on_gpu_tree} on the GPU's own tree)")
    assert sc.verify_passes_compared >= 1
    if fused_chain:
        say(f"{name}: {sc.steps_without_draft_pass} step(s) built their tree from in-pass drafts")
        assert sc.steps_without_draft_pass >= 1
    sc.gpu.close()


@pytest.mark.parametrize("tree_size", [1, 16, 32, 64, 128])
def test_llama13b_width_tree_size_sweep(tree_size):
    _shallow_case("llama13b", 96, tree_size=tree_size)


def test_llama13b_width_at_the_full_cache_length():
    """Config 4 at its own cache length: 2048 cached tokens (the key-slice paths of both attention kernels), T = 64."""
    _shallow_case("llama13b", 2048, cache=2048 + 2 * 64 + 16)


def test_llama70b_width_at_the_full_cache_length():
    """Config 5 at its own cache length: 64 query heads on 8 key/value heads over 4096 cached tokens (the ring attention
    kernel with grouped heads, in the verify pass and in the draft pass of 4 rows), 2 layers, T = 64."""
    _shallow_case("llama70b", 4096, cache=4096 + 2 * 64 + 16)


@pytest.mark.parametrize("fused_chain", [False, True])
def test_llama13b_width_with_a_transfer_layer_per_step(fused_chain):
    """The 13B setting of Sec. 4.1 has one transfer layer per step (25 / 30 / 35 of 40): here the 13B widths at 4 layers
    with the steps' maps after layers 1 / 2 / 3, so pseudo rows join the draft pass, or the verify pass, at three
    different blocks; drafting after acceptance and with the rank-0 chain drafting in the pass."""
    _shallow_case("llama13b_t253035", 96, fused_chain=fused_chain, steps=2, layers=4, transfer_layers=(1, 2, 3))


def test_llama70b_width_grouped_query_attention():
    _shallow_case("llama70b", 80)


@pytest.mark.parametrize("name,prompt_len", [("llama7b", 96), ("llama70b", 80)])
def test_wide_bf16_drafting_inside_the_verify_pass(name, prompt_len):
    """64-node tree plus k pseudo rows under each node of the rank-0 chain (76 or 84 rows: the 80- and 96-row
    product instances, two row groups in the tiled attention), three steps."""
    _shallow_case(name, prompt_len, fused_chain=True, steps=3)


def test_llama7b_width_two_layers_against_oracle():
    """Full 7B widths (d 4096, 32x128 heads, FFN 11008, vocab 32000), 64-node tree, cache 512, the launch
    configuration the benchmark times; depth cut to 2 layers so the fp64 oracle finishes in seconds."""
    H = _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), prompt_len=512, max_cache=640)
    say("7B-width 2 layers: generating weights")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    say("7B-width 2 layers: oracle + gpu")
    sc = H.StepCompare(wl, tensors_gpu=tensors, tensors_cpu=cpu_tensors)
    sc.check_prefill()
    r = sc.step(require_same_tokens=False)
    say(f"7B-width 2 layers: emitted {r['emitted']} oracle {r['oracle']['emitted']}, verify passes compared "
        f"{sc.verify_passes_compared}, worst logit error / bound {sc.max_err:.3f}, element-wise with rms floor "
        f"{sc.max_elementwise:.3f} x")
    assert sc.verify_passes_compared == 1
    sc.gpu.close()


@pytest.mark.parametrize("vocab", [33000, 50000, 140000])
def test_candidate_selection_on_large_vocabularies(vocab):
    """Vocabularies past 32768 use the sixteen-entries-per-lane instance of the candidate selection, past 131072 its
    block-wide fallback: three steps of a very small model, candidates and tokens against the oracle's rule."""
    H = _H()
    wl = small_workload(name=f"vocab{vocab}", n_layers=2, d_model=64, n_heads=2, n_kv_heads=1, head_dim=32, d_ffn=72,
                        vocab=vocab, k=2, transfer_layers=(1, 1), prompt_len=9, max_cache=64, tree_size=12,
                        branching=(5, 4), seed=31 + vocab)
    say(f"large vocabulary {vocab}")
    sc = H.StepCompare(wl)
    sc.check_prefill()
    out = []
    for step in range(3):
        out += sc.step()["emitted"]
    assert out == sc.model.ar_greedy(sc.prompt, len(out))
    sc.gpu.close()
