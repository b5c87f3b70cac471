#!/usr/bin/env python3
"""Benchmark of the Hidden Transfer tree-verify decode step on one MI355X.

A "step" is one pass of the whole hot path on the Llama-2-7B-shaped workload (bf16, batch 1, 512-token
cache, 64-node tree): hidden transfer -> draft pass of the k pseudo rows -> top-k -> tree build ->
tree-verify forward -> greedy acceptance -> KV compaction.  Weights and prompt are seeded synthetic data
already resident in HBM when timing starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def model_bytes(wl, T, n):
    """Algorithmic HBM bytes of one verify pass: every weight once, KV cache read once, new KV written."""
    es = 2 if wl.dtype == "bf16" else 4
    d, qd, kvd, f, v = wl.d_model, wl.n_heads * wl.head_dim, wl.n_kv_heads * wl.head_dim, wl.d_ffn, wl.vocab
    per_layer = (d * (qd + 2 * kvd) + qd * d + 3 * d * f + 2 * d) * es
    weights = wl.n_layers * per_layer + (v * d + d) * es + T * d * es        # + embedding rows actually read
    kv_read = wl.n_layers * 2 * (n + T) * kvd * es
    kv_write = wl.n_layers * 2 * T * kvd * es
    return weights + kv_read + kv_write


def cpu_baseline(wl, T, n, weights):
    """Times the fp64 oracle on one decoder block + the LM head at the real shape and extrapolates.
    `weights` are the seeded tensors already generated on the GPU; layer 0 and the head are copied to the host."""
    import numpy as np
    from oracle import ht_oracle as O
    tens = {}
    for name, val in weights.items():
        tens[name] = [val[0].cpu(), val[0].cpu()] if isinstance(val, list) and name != "w_transfer" else (
            [t.cpu() for t in val] if isinstance(val, list) else val.cpu())
    cfg = O.OracleConfig(2, wl.d_model, wl.n_heads, wl.n_kv_heads, wl.head_dim, wl.d_ffn, wl.vocab, wl.k,
                         tuple(1 for _ in range(wl.k)), wl.rms_eps, wl.rope_base)
    model = O.OracleModel(cfg, O.OracleWeights(tens))
    rng = np.random.default_rng(0)
    x = rng.normal(size=(T, wl.d_model))
    kc = rng.normal(size=(n, wl.n_kv_heads, wl.head_dim))
    vc = rng.normal(size=(n, wl.n_kv_heads, wl.head_dim))
    pos = np.full(T, n)
    vis_old = np.ones((T, n), dtype=bool)
    vis_new = np.tril(np.ones((T, T), dtype=bool))
    model.block(0, x[:2], pos[:2], kc, vc, vis_old[:2], vis_new[:2, :2])      # warm the BLAS threads
    kx = x[:wl.k]

    def sample():
        t0 = time.perf_counter()
        y, _, _ = model.block(0, x, pos, kc, vc, vis_old, vis_new)
        t1 = time.perf_counter()
        model.logits(y)
        t2 = time.perf_counter()
        model.block(0, kx, pos[:wl.k], kc, vc, vis_old[:wl.k], vis_new[:wl.k, :wl.k])
        t3 = time.perf_counter()
        model.logits(kx)
        t4 = time.perf_counter()
        return t1 - t0, t2 - t1, t3 - t2, t4 - t3

    sample()                                                # first call pays page faults and thread start-up
    acc = [0.0, 0.0, 0.0, 0.0]
    reps = 0
    while sum(acc) < 15.0 and reps < 2000:                   # about 15 s of CPU work
        for i, t in enumerate(sample()):
            acc[i] += t
        reps += 1
    t_block, t_head, t_dblock, t_dhead = (a / reps for a in acc)
    cpu_work = sum(acc)
    draft_blocks = sum(wl.n_layers - t for t in wl.transfer_layers) / wl.k      # a k-row block, averaged over the joins
    est = wl.n_layers * t_block + t_head + draft_blocks * t_dblock + t_dhead
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": round(est * 1e3, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "sample": (f"fp64 numpy oracle, one of {wl.n_layers} decoder blocks at T={T} rows and n={n} cached keys plus "
                       f"the LM head, and one draft block at {wl.k} rows, mean of {reps} repetitions "
                       f"({cpu_work:.1f} s of CPU work) extrapolated to a full step "
                       f"({wl.n_layers} verify blocks + head + {draft_blocks:g} draft blocks + head)")}


def time_dominant_kernel(wl, T, dev, tdt, stream, calibrate=False):
    """The fused gate/up projection act = silu(a . Wg^T) * (a . Wu^T), the kernel the pass spends most of its time in,
    timed alone through its own entry point with HIP events on the launch stream, over rotating packed weight copies
    (4 x 180 MB > 256 MB of last-level cache)."""
    import torch
    from ht_inputs import counter_normal
    import paper_2404_12022_amd.binding as B
    M, N, K = T, 2 * wl.d_ffn, wl.d_model
    copies = 4
    a = counter_normal(wl.seed, 899, (B.ht_padded_rows(M), K), 1.0, device=dev, dtype=tdt)
    f = wl.d_ffn
    out = torch.empty(M, f, dtype=tdt, device=dev)
    packed = []
    for i in range(copies):                      # same streaming layout ht_init_model gives the model's weights
        wg = counter_normal(wl.seed, 900 + 2 * i, (f, K), 0.02, device=dev, dtype=tdt)
        wu = counter_normal(wl.seed, 901 + 2 * i, (f, K), 0.02, device=dev, dtype=tdt)
        p = torch.empty(B.ht_weight_pack_bytes(N, K), dtype=torch.uint8, device=dev)
        B.ht_gate_up_pack(wg, wu, f, K, p)
        torch.cuda.synchronize()
        packed.append(p)
        del wg, wu
    for i in range(copies):
        B.ht_gate_up_silu_packed(a, packed[i], M, f, K, out)
    launches = 40
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(launches):
        B.ht_gate_up_silu_packed(a, packed[i % copies], M, f, K, out)
    e1.record(stream)
    e1.synchronize()
    ms_kernel = e0.elapsed_time(e1) / launches
    # the same buffers read once by a kernel that only streams (same access pattern, no arithmetic): what the
    # memory system delivers to a launch of this size
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    got = 0
    for i in range(copies):
        got = B.ht_stream_read_probe(packed[i], sink)
    e0.record(stream)
    for i in range(launches):
        B.ht_stream_read_probe(packed[i % copies], sink)
    e1.record(stream)
    e1.synchronize()
    stream_gbps = got / (e0.elapsed_time(e1) / launches * 1e-3) / 1e9
    if calibrate:                                # a plain device copy of known size, for scaling the HBM counters
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    kernel_bytes = N * K * 2 + M * K * 2 + M * f * 2        # weights + activation panel in, bf16 activations out
    return {"M": M, "N": N, "K": K, "ms": ms_kernel, "bytes": kernel_bytes, "stream_GBps": stream_gbps}


def time_attention_op(dev):
    """ht_tree_attention at the op workload: bf16, 32 query heads x 128, KV cache 4096 + 128 tree rows, random tree of
    depth <= 6, rotary + append + attention per call, eight rotating cache copies (8 x 69 MB > last-level cache)."""
    import torch
    from ht_inputs import counter_normal, random_tree
    from ht_inputs.workloads import ATTENTION_OP as A
    import paper_2404_12022_amd.binding as B
    T, n, Hq, Hkv, hd = A["tree_size"], A["cache_len"], A["n_heads"], A["n_kv_heads"], A["head_dim"]
    cap = n + T
    parent, _ = random_tree(A["seed"], T, A["max_depth"])
    bf = torch.bfloat16
    q = counter_normal(A["seed"], 21, (T, Hq, hd), 1.0, device=dev, dtype=bf)
    kn = counter_normal(A["seed"], 24, (T, Hkv, hd), 1.0, device=dev, dtype=bf)
    vn = counter_normal(A["seed"], 25, (T, Hkv, hd), 1.0, device=dev, dtype=bf)
    copies = 8
    kcs = [counter_normal(A["seed"], 100 + i, (cap, Hkv, hd), 1.0, device=dev, dtype=bf) for i in range(copies)]
    vcs = [counter_normal(A["seed"], 200 + i, (Hkv, hd, cap), 1.0, device=dev, dtype=bf) for i in range(copies)]
    out = torch.empty(T, Hq * hd, dtype=bf, device=dev)
    scratch = torch.empty(B.ht_tree_attention_scratch_bytes(T, Hq, hd), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def call(i, tree=parent):
        B.ht_tree_attention(q, kn, vn, kcs[i % copies], vcs[i % copies], cap, n, T, tree, Hq, Hkv, hd, B.HT_BF16,
                            A["rope_base"], out, scratch)

    def timed(tree):
        for i in range(copies):
            call(i, parent)                       # also leaves the tree tables in `scratch`
        reps = 40
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(reps):
            call(i, tree)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps

    us_upload = timed(parent)                     # every call builds and uploads the tree tables
    us = timed(None)                              # the tables of the static tree stay in scratch
    by = 2 * cap * Hkv * hd * 2 + 2 * T * Hq * hd * 2 + 2 * T * Hkv * hd * 2 * 2
    return {"op": "ht_tree_attention", "T": T, "cache_len": n, "heads": Hq, "head_dim": hd, "us_per_call": round(us, 2),
            "us_per_call_with_tree_upload": round(us_upload, 2),
            "algorithmic_bytes": by, "GBps": round(by / (us * 1e-6) / 1e9, 1),
            "frac_of_hbm_peak": round(by / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "note": "per call: rotary table + rotary/append kernel + attention kernel + slice merge kernel; the "
                    "static tree's tables are uploaded once"}


def time_second_workload(name, dev, tree_sizes, reps, also_layers=None):
    """Verify pass of another named workload at its own cache length: one model, a sweep over tree sizes (HIP events
    on the launch stream), the one-token pass, and the whole step at the workload's own tree size in two schedules."""
    import torch
    from ht_inputs import WORKLOADS, make_weights, counter_tokens, prune_tree
    from ht_inputs.generators import PROMPT_STREAM
    import paper_2404_12022_amd.binding as B
    wl = WORKLOADS[name]
    T0, n0 = wl.tree_size, wl.prompt_len
    steps = 10
    rows = max(tree_sizes + [T0 + (wl.k + 1) * wl.k])
    wl = wl.with_(max_cache=(n0 + 4 * (2 * steps + 8) * (wl.k + 1) + rows + 7) // 8 * 8)
    tdt = torch.bfloat16
    param_bytes = 2 * wl.n_layers * (wl.d_model * (wl.n_heads + 2 * wl.n_kv_heads) * wl.head_dim +
                                     wl.n_heads * wl.head_dim * wl.d_model + 3 * wl.d_model * wl.d_ffn)
    if param_bytes > 100e9:                      # too large for the original and the packed copy together: layer by layer
        from ht_inputs import layer_weights
        weights = make_weights(wl, wl.seed, dev, tdt, layers=[])
        head = weights["lm_head"]
        weights["lm_head"] = None
        model = B.HTModel(B.make_config(wl, max_tree=min(128, rows)), weights, dev)
        for layer in range(wl.n_layers):
            lw = layer_weights(wl, wl.seed, layer, dev, tdt)
            model.ht_load_layer(layer, lw)
            torch.cuda.synchronize()
            del lw
        model.ht_load_lm_head(head)
        torch.cuda.synchronize()
        del head
    else:
        weights = make_weights(wl, wl.seed, dev, tdt)
        model = B.HTModel(B.make_config(wl, max_tree=min(128, rows)), weights, dev)
    prompt = [int(t) for t in counter_tokens(wl.seed, PROMPT_STREAM, n0, wl.vocab)]
    parent, rank = prune_tree(wl.branching, T0)
    model.ht_set_tree(parent, rank)
    model.ht_prefill(prompt)
    stream = torch.cuda.current_stream()

    def verify_ms(tp, tr):
        model.ht_set_tree(tp, tr)
        toks = torch.tensor(prompt[:len(tp)], dtype=torch.int32, device=dev)
        for _ in range(3):
            model.ht_tree_verify_step(toks)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            model.ht_tree_verify_step(toks)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    def step_ms(nodes, model=model):
        model.ht_set_tree(parent, rank)
        model.ht_set_fused_nodes(nodes)
        for _ in range(3):
            model.ht_transfer(); model.ht_tree_verify_step(); model.ht_accept_and_compact()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            model.ht_transfer(); model.ht_tree_verify_step(); model.ht_accept_and_compact()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    ms_one = verify_ms([-1], [0])
    sweep = []
    for ts in tree_sizes:
        tp, tr = prune_tree(wl.branching, ts)
        ms_t = verify_ms(tp, tr)
        by = model_bytes(wl, ts, n0)
        sweep.append({"T": ts, "verify_pass_ms": round(ms_t, 4), "verify_over_one_token": round(ms_t / ms_one, 4),
                      "hbm_GBps": round(by / (ms_t * 1e-3) / 1e9, 1),
                      "hbm_frac_of_peak": round(by / (ms_t * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
    chain, cur = [0], 0
    while True:
        kids = [v for v in range(T0) if parent[v] == cur and rank[v] == 0]
        if not kids:
            break
        cur = kids[0]
        chain.append(cur)
    ms_s1 = step_ms([])
    ms_hybrid = step_ms(chain)
    res = {"workload": f"{wl.name}: {wl.n_layers} layers d={wl.d_model} {wl.n_heads}x{wl.head_dim} heads ffn={wl.d_ffn}, "
                       f"cache {n0}, k={wl.k} transfer after layer {sorted(set(wl.transfer_layers))}",
           "one_token_step_ms": round(ms_one, 4), "tree_size_sweep": sweep, "tree_size_of_the_steps": T0,
           "step_ms_draft_after_accept": round(ms_s1, 4), "step_ms_rank0_chain_drafts_in_verify_pass": round(ms_hybrid, 4)}
    model.close()
    del model
    torch.cuda.empty_cache()
    if also_layers:        # the same decoder with one transfer layer per step (the 13B setting of Sec. 4.1)
        wl2 = wl.with_(transfer_layers=tuple(also_layers))
        m2 = B.HTModel(B.make_config(wl2, max_tree=min(128, rows)), weights, dev)
        m2.ht_set_tree(parent, rank)
        m2.ht_prefill(prompt)
        res["transfer_after_layers_%s" % "_".join(str(t) for t in also_layers)] = {
            "step_ms_draft_after_accept": round(step_ms([], m2), 4),
            "step_ms_rank0_chain_drafts_in_verify_pass": round(step_ms(chain, m2), 4)}
        m2.close()
        del m2
    del weights
    torch.cuda.empty_cache()
    return res


def measured_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "gemm_gateup_hbm_traffic.json")
    try:
        with open(path) as fh:
            return json.load(fh)["hbm_bytes_per_launch"]
    except Exception:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama7b")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tree-sizes", default="",
                    help="comma-separated tree sizes: adds a `sweep` list of verify-pass latencies at the same cache")
    ap.add_argument("--cache-lens", default="",
                    help="comma-separated cache lengths: adds a `cache_sweep` list (verify and one-token pass after a "
                         "prefill of that many random tokens)")
    ap.add_argument("--fused-counts", default="",
                    help="comma-separated numbers of tree nodes (taken in node order) that carry pseudo rows in the "
                         "verify pass: adds a `fused_sweep` list of verify-pass latencies")
    ap.add_argument("--k-values", default="",
                    help="comma-separated numbers of transfer steps k (= tree depth) to time the step at, same T: "
                         "a fresh model per value (transfer maps for k steps at the workload's first transfer layer, "
                         "tree prune_tree([10] * k, T))")
    ap.add_argument("--training-forward", type=int, default=0, metavar="N",
                    help="also time the forward pass of the training stage with its KL loss over N tokens for the "
                         "first transfer step (`training_forward` object)")
    ap.add_argument("--attention-op", action="store_true",
                    help="time the tree-attention op alone (32 heads x 128, cache 4096, random 128-node tree)")
    ap.add_argument("--only-main", action="store_true",
                    help="skip the objects a default run adds to the 7B line: the tree-attention op and the 13B workload")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the HIP-graph launch medians (counter collection under rocprofv3 does not survive graph launches)")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant-kernel loop plus a device copy of known size (for rocprofv3 runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from ht_inputs import WORKLOADS, make_weights, counter_tokens, prune_tree, counter_normal
    from ht_inputs.generators import PROMPT_STREAM
    import paper_2404_12022_amd.binding as B

    dev = "cuda:0"
    wl = WORKLOADS[args.workload]
    if args.attention_op:
        print(json.dumps(time_attention_op(dev)))
        return
    if args.roofline_only:
        tdt0 = torch.bfloat16
        k = time_dominant_kernel(wl, wl.tree_size, dev, tdt0, torch.cuda.current_stream(), calibrate=True)
        print(json.dumps({"kernel_ms": k["ms"], "bytes": k["bytes"], "GBps": k["bytes"] / (k["ms"] * 1e-3) / 1e9}))
        return
    sweep_sizes = [int(t) for t in args.tree_sizes.split(",") if t]
    cache_lens = [int(t) for t in args.cache_lens.split(",") if t]
    fused_counts = [int(t) for t in args.fused_counts.split(",") if t]
    fused_rows = max([wl.k + 1] + fused_counts) * wl.k   # pseudo rows under the rank-0 chain (or the largest sweep entry)
    headroom = 5 * (args.steps + args.warmup + 4) * (wl.k + 1) + max([wl.tree_size * (1 + wl.k)] + sweep_sizes)
    if args.training_forward:
        sweep_sizes_model = sweep_sizes + [128]      # 128-row passes: 63 positions, their pseudo rows, one of lookahead
    else:
        sweep_sizes_model = sweep_sizes
    wl = wl.with_(max_cache=(max([wl.prompt_len, args.training_forward] + cache_lens) + headroom + 7) // 8 * 8)
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    T, n0 = wl.tree_size, wl.prompt_len
    parent, rank = prune_tree(wl.branching, T)
    prompt = [int(t) for t in counter_tokens(wl.seed, PROMPT_STREAM, n0, wl.vocab)]
    param_bytes = 2 * wl.n_layers * (wl.d_model * (wl.n_heads + 2 * wl.n_kv_heads) * wl.head_dim +
                                     wl.n_heads * wl.head_dim * wl.d_model + 3 * wl.d_model * wl.d_ffn)
    if param_bytes > 100e9:
        # too large to hold the original and the packed copy together: supply one layer at a time
        from ht_inputs import layer_weights
        weights = make_weights(wl, wl.seed, dev, tdt, layers=[])
        head = weights["lm_head"]
        weights["lm_head"] = None
        model = B.HTModel(B.make_config(wl, max_tree=min(128, max([T + fused_rows] + sweep_sizes_model))), weights, dev)
        for layer in range(wl.n_layers):
            lw = layer_weights(wl, wl.seed, layer, dev, tdt)
            model.ht_load_layer(layer, lw)
            torch.cuda.synchronize()
            del lw
        model.ht_load_lm_head(head)
        torch.cuda.synchronize()
        del head
    else:
        weights = make_weights(wl, wl.seed, dev, tdt)
        full_rows = T * (1 + wl.k)                   # every node with its k pseudo rows: the paper's own schedule
        rows_model = max([T + fused_rows] + sweep_sizes_model + ([full_rows] if full_rows <= B.HT_MAX_ROWS else []))
        model = B.HTModel(B.make_config(wl, max_tree=min(B.HT_MAX_ROWS, rows_model)), weights, dev)
    model.ht_set_tree(parent, rank)
    model.ht_prefill(prompt)
    stream = torch.cuda.current_stream()

    def full_step():
        model.ht_transfer()
        model.ht_tree_verify_step()
        return model.ht_accept_and_compact()

    # ---- whole hot path, K steps, wall clock bracketed by synchronisation.  Timed in both schedules: drafting
    # after acceptance (transfer + draft pass + verify pass per step), and drafting inside the verify pass for
    # the nodes of the rank-0 chain (k pseudo rows under each; a step whose acceptance ends on that chain needs
    # no transfer and no draft pass, any other step falls back to the first schedule).  `value` is the second.
    def timed_steps():
        acc = 0
        for _ in range(args.warmup):
            full_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            acc += full_step()[0]
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps, acc

    ms_step_s1, _ = timed_steps()
    # the same schedule with the cache length kept on the device: K steps enqueued at once, one host wait at the end
    loop_steps = min(args.steps, B.HT_MAX_LOOP_STEPS)
    model.ht_decode_steps(min(max(args.warmup, 1), B.HT_MAX_LOOP_STEPS))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model.ht_decode_steps(loop_steps)
    torch.cuda.synchronize()
    ms_step_loop = (time.perf_counter() - t0) * 1e3 / loop_steps
    # the same schedule with the tree chosen anew at every step among the best candidates of every pseudo position
    dyn_b = wl.branching[0]
    model.ht_set_dynamic_tree(T, dyn_b)
    ms_step_dynamic, _ = timed_steps()
    model.ht_set_tree(parent, rank)
    chain, cur = [0], 0
    while True:
        kids = [v for v in range(T) if parent[v] == cur and rank[v] == 0]
        if not kids:
            break
        cur = kids[0]
        chain.append(cur)
    model.ht_set_fused_nodes(chain)
    ms_step, accepted = timed_steps()
    # the paper's own schedule: every node carries its k pseudo rows, T (1 + k) rows above the transfer layer
    ms_step_full = None
    if T * (1 + wl.k) <= model.cfg.max_tree:
        model.ht_set_fused_nodes(list(range(T)))
        ms_step_full, _ = timed_steps()
    model.ht_set_fused_nodes([])

    # ---- verify pass alone (explicit tokens, no draft) and the one-token step, HIP events on the launch stream
    def time_verify(tree_parent, tree_rank, reps):
        model.ht_set_tree(tree_parent, tree_rank)
        toks = torch.tensor(prompt[:len(tree_parent)], dtype=torch.int32, device=dev)
        for _ in range(3):
            model.ht_tree_verify_step(toks)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            model.ht_tree_verify_step(toks)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    # ---- the same pass captured once in a HIP graph: median of 100 single launches after 20 warm-up launches
    def time_verify_graph(tree_parent, tree_rank, launches=100, warm=20):
        model.ht_set_tree(tree_parent, tree_rank)
        toks = torch.tensor(prompt[:len(tree_parent)], dtype=torch.int32, device=dev)
        model.ht_tree_verify_step(toks)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            model.ht_tree_verify_step(toks)
        for _ in range(warm):
            graph.replay()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
        for a, b in ev:
            a.record(stream)
            graph.replay()
            b.record(stream)
        torch.cuda.synchronize()
        ts_ = sorted(a.elapsed_time(b) for a, b in ev)
        del graph
        return ts_[len(ts_) // 2]

    n_now = model.ht_cache_len()
    reps = max(5, args.steps)
    ms_verify = time_verify(parent, rank, reps)
    ms_one = time_verify([-1], [0], reps)
    ms_verify_graph = ms_one_graph = None
    if not args.no_graph:
        ms_verify_graph = time_verify_graph(parent, rank)
        ms_one_graph = time_verify_graph([-1], [0])
    sweep = []
    for ts in sweep_sizes:
        tp, tr = prune_tree(wl.branching, ts)
        ms_t = time_verify(tp, tr, reps)
        by = model_bytes(wl, ts, n_now)
        sweep.append({"T": ts, "verify_pass_ms": round(ms_t, 4), "hbm_GBps": round(by / (ms_t * 1e-3) / 1e9, 1),
                      "hbm_frac_of_peak": round(by / (ms_t * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
    model.ht_set_tree(parent, rank)
    fused_sweep = []
    for cnt in fused_counts:                     # verify pass with explicit tokens and `cnt` nodes drafting in-pass
        if T + cnt * wl.k > model.cfg.max_tree:
            continue
        model.ht_set_tree(parent, rank)
        model.ht_set_fused_nodes(list(range(cnt)))
        toks = torch.tensor(prompt[:T], dtype=torch.int32, device=dev)
        for _ in range(3):
            model.ht_tree_verify_step(toks)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            model.ht_tree_verify_step(toks)
        e1.record(stream)
        e1.synchronize()
        fused_sweep.append({"fused_nodes": cnt, "rows_in_upper_blocks": T + cnt * wl.k,
                            "verify_pass_ms": round(e0.elapsed_time(e1) / reps, 4)})
    model.ht_set_tree(parent, rank)
    cache_sweep = []
    for n_c in cache_lens:
        long_prompt = [int(t) for t in counter_tokens(wl.seed, PROMPT_STREAM, n_c, wl.vocab)]
        model.ht_prefill(long_prompt)
        ms_v = time_verify(parent, rank, max(5, args.steps // 2))
        ms_1 = time_verify([-1], [0], max(5, args.steps // 2))
        by = model_bytes(wl, T, n_c)
        cache_sweep.append({"cache_len": n_c, "verify_pass_ms": round(ms_v, 4), "one_token_step_ms": round(ms_1, 4),
                            "verify_over_one_token": round(ms_v / ms_1, 4),
                            "verify_hbm_GBps": round(by / (ms_v * 1e-3) / 1e9, 1),
                            "kv_read_share_of_bytes": round(1 - model_bytes(wl, T, 0) / by, 4)})
    model.ht_set_tree(parent, rank)

    # ---- the step against the number of transfer steps k = depth of the tree, T fixed (a model per value: the
    # same decoder weights, k transfer maps, a k-level tree; both schedules as above)
    depth_sweep = []
    for kk in [int(t) for t in args.k_values.split(",") if t]:
        if param_bytes > 100e9:
            break
        wl_k = wl.with_(k=kk, transfer_layers=(wl.transfer_layers[0],) * kk, branching=(10,) * kk)
        w_k = dict(weights)
        w_k["w_transfer"] = make_weights(wl_k, wl.seed, dev, tdt, layers=[])["w_transfer"]
        p_k, r_k = prune_tree(wl_k.branching, T)
        chain_k, cur = [0], 0
        while True:
            kids = [v for v in range(T) if p_k[v] == cur and r_k[v] == 0]
            if not kids:
                break
            cur = kids[0]
            chain_k.append(cur)
        m_k = B.HTModel(B.make_config(wl_k, max_tree=min(128, T + len(chain_k) * kk)), w_k, dev)
        m_k.ht_set_tree(p_k, r_k)
        m_k.ht_prefill(prompt)
        row = {"k": kk, "tree_depth": max(len(chain_k) - 1, 0)}
        for label, nodes in (("step_ms_draft_after_accept", []), ("step_ms_draft_in_verify_pass", chain_k)):
            m_k.ht_set_fused_nodes(nodes)
            for _ in range(args.warmup):
                m_k.ht_transfer(); m_k.ht_tree_verify_step(); m_k.ht_accept_and_compact()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                m_k.ht_transfer(); m_k.ht_tree_verify_step(); m_k.ht_accept_and_compact()
            torch.cuda.synchronize()
            row[label] = round((time.perf_counter() - t0) * 1e3 / args.steps, 4)
        row["pseudo_rows_in_verify_pass"] = len(chain_k) * kk
        depth_sweep.append(row)
        m_k.close()
        del m_k, w_k
        torch.cuda.empty_cache()

    # ---- forward pass of the training stage (Sec. 3.3) over N tokens, first transfer step: chunks of
    # (max_tree - 1) / 2 positions; the blocks above the transfer layer and the LM head are walked once per chunk,
    # the blocks below it once per two chunks
    def time_training_forward(model, n_tr):
        step_tr = 1
        toks_tr = [int(t) for t in counter_tokens(wl.seed, PROMPT_STREAM, n_tr, wl.vocab)]
        model.ht_training_forward(step_tr, toks_tr)
        reps_tr = 3
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps_tr):
            _, loss_tr = model.ht_training_forward(step_tr, toks_tr)
        ms_tr = (time.perf_counter() - t0) * 1e3 / reps_tr
        chunk = (min(model.cfg.max_tree, B.HT_MAX_TREE) - step_tr) // 2
        passes = (n_tr + chunk - 1) // chunk
        t_layer = wl.transfer_layers[step_tr - 1]
        per_layer = 2 * (wl.d_model * (wl.n_heads + 2 * wl.n_kv_heads) * wl.head_dim + wl.n_heads * wl.head_dim * wl.d_model +
                         3 * wl.d_model * wl.d_ffn)                       # bytes of one block's matrices (bf16)
        head = 2 * wl.vocab * wl.d_model
        passes_low = (n_tr + 2 * chunk - 1) // (2 * chunk)
        byts = passes_low * t_layer * per_layer + passes * ((wl.n_layers - t_layer) * per_layer + head)   # K/V reads left out
        pseudo_rows = n_tr - step_tr + 1
        rows_low, rows_up = n_tr + passes_low * step_tr, n_tr + passes * step_tr + pseudo_rows     # lookahead rows run twice
        flops = per_layer * (t_layer * rows_low + (wl.n_layers - t_layer) * rows_up) + head * rows_up   # 2 flops per bf16 weight byte / 2
        training = {"tokens": n_tr, "transfer_step": step_tr, "ms": round(ms_tr, 3), "tokens_per_s": round(n_tr / (ms_tr * 1e-3), 1),
                    "passes_upper_blocks": passes, "passes_lower_blocks": passes_low, "positions_per_pass": chunk,
                    "loss": loss_tr,
                    "weight_bytes_streamed": byts, "hbm_GBps": round(byts / (ms_tr * 1e-3) / 1e9, 1),
                    "hbm_frac_of_peak": round(byts / (ms_tr * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "matrix_TFLOPs": round(flops / (ms_tr * 1e-3) / 1e12, 1),
                    "matrix_frac_of_bf16_peak": round(flops / (ms_tr * 1e-3) / 2.5e15, 4)}
        # the same forward pass with all positions in one pass per block (token-tiled products)
        ws_bytes = B.C.c_size_t(0)
        B._check(B.lib.ht_training_workspace_bytes(B.C.byref(model.cfg), n_tr, B.C.byref(ws_bytes)))
        ws_tr = torch.empty(ws_bytes.value, dtype=torch.uint8, device=dev)
        _, loss_b = model.ht_training_forward_batched(step_tr, toks_tr, workspace=ws_tr)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps_tr):
            model.ht_training_forward_batched(step_tr, toks_tr, workspace=ws_tr)
        ms_b = (time.perf_counter() - t0) * 1e3 / reps_tr
        rows_b_low, rows_b_up = n_tr, n_tr + pseudo_rows
        flops_b = per_layer * (t_layer * rows_b_low + (wl.n_layers - t_layer) * rows_b_up) + head * rows_b_up \
            + 2 * wl.d_model * wl.d_model * pseudo_rows
        training["batched"] = {"ms": round(ms_b, 3), "tokens_per_s": round(n_tr / (ms_b * 1e-3), 1), "loss": loss_b,
                               "matrix_TFLOPs": round(flops_b / (ms_b * 1e-3) / 1e12, 1),
                               "matrix_frac_of_bf16_peak": round(flops_b / (ms_b * 1e-3) / 2.5e15, 4),
                               "workspace_bytes": ws_bytes.value,
                               "note": "every projection once over all rows (token-tiled kernel); attention: one causal launch per block for the hidden rows, one for the pseudo rows"}
        # what the matrix cores of this machine sustain on register operands alone, per instruction form
        sink_m = torch.zeros(1, dtype=torch.int32, device=dev)
        rates = {}
        for form, name in ((0, "v_mfma_f32_16x16x32_bf16"), (1, "v_mfma_f32_32x32x16_bf16"),
                           (2, "v_mfma_f32_16x16x32_bf16, hashed operand bits"),
                           (3, "v_mfma_f32_32x32x16_bf16, hashed operand bits")):
            B.ht_mfma_rate_probe(form, 2000, sink_m)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fl = sum(B.ht_mfma_rate_probe(form, 2000, sink_m) for _ in range(5))
            e1.record(stream)
            e1.synchronize()
            rates[name] = round(fl / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
        training["measured_matrix_core_TFLOPs"] = rates
        training["batched"]["matrix_frac_of_measured_16x16x32_rate"] = round(
            flops_b / (ms_b * 1e-3) / 1e12 / rates["v_mfma_f32_16x16x32_bf16, hashed operand bits"], 4)
        del ws_tr
        return training


    training = None
    if args.training_forward:
        training = time_training_forward(model, args.training_forward)
        model.ht_prefill(prompt)

    kern = time_dominant_kernel(wl, T, dev, tdt, stream)
    achieved = kern["bytes"] / (kern["ms"] * 1e-3) / 1e9
    verify_bytes = model_bytes(wl, T, n_now)
    one_bytes = model_bytes(wl, 1, n_now)
    res = {
        "metric": "tree_verify_step_latency_ms", "value": round(ms_step, 4), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_layers} layers d={wl.d_model} {wl.n_heads}x{wl.head_dim} heads "
                               f"ffn={wl.d_ffn} vocab={wl.vocab}, batch 1, cache {n0}, tree T={T} {list(wl.branching)}, "
                               f"k={wl.k} transfer after layer {sorted(set(wl.transfer_layers))}; step = hidden transfer + pseudo "
                               f"rows through the upper blocks + top-k + tree build + verify + accept + compact.  "
                               f"Schedule of `value`: the pseudo rows of the rank-0 chain ({len(chain)} nodes x k rows) ride in "
                               f"the verify pass and, with random maps, every acceptance ends on that chain, so no step "
                               f"needs a draft pass: the hybrid's best case.  The schedule that drafts after every "
                               f"acceptance costs `step_ms_draft_after_accept`, the paper's own schedule (all {T} nodes "
                               f"draft in the pass) `step_ms_every_node_drafts_in_verify_pass`"},
        "step_ms_draft_after_accept": round(ms_step_s1, 4),
        "step_ms_every_node_drafts_in_verify_pass": None if ms_step_full is None else round(ms_step_full, 4),
        "step_ms_draft_after_accept_device_resident_loop": round(ms_step_loop, 4),
        "step_ms_draft_after_accept_dynamic_tree": {"ms": round(ms_step_dynamic, 4), "candidates_per_position": dyn_b},
        "verify_pass_ms": round(ms_verify, 4), "one_token_step_ms": round(ms_one, 4),
        "verify_over_one_token": round(ms_verify / ms_one, 4),
        "graph_launch_median": None if ms_verify_graph is None else {
            "verify_pass_ms": round(ms_verify_graph, 4), "one_token_step_ms": round(ms_one_graph, 4),
            "verify_over_one_token": round(ms_verify_graph / ms_one_graph, 4), "launches": 100, "warmup_launches": 20},
        "candidate_tokens_per_s": round(T / (ms_verify * 1e-3), 1),
        "accepted_tokens_per_step": round(accepted / args.steps, 3),
        "verify_hbm_GBps": round(verify_bytes / (ms_verify * 1e-3) / 1e9, 1),
        "verify_hbm_frac_of_peak": round(verify_bytes / (ms_verify * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "one_token_hbm_GBps": round(one_bytes / (ms_one * 1e-3) / 1e9, 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic() if wl.name == "llama7b" else None,
                     "traffic_source": "FETCH_SIZE + WRITE_SIZE of this kernel from the committed rocprofv3 counter runs "
                                       "(profiles/gemm_packed_gateup_7b_hbm_counters.md), not a counter read in this run",
                     "whole_verify_pass": {"achieved": round(verify_bytes / (ms_verify * 1e-3) / 1e9, 1),
                                           "frac": round(verify_bytes / (ms_verify * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                           "bytes": verify_bytes, "ms": round(ms_verify, 4)},
                     "kernel": (("gemm_packed_kernel<MT=4,R=2,WAVES=3,EPI_SILU,KC=128>" if (kern["N"] // 16 + 5) // 6 <= 260
                                 else "gemm_packed_kernel<MT=4,R=2,WAVES=4,EPI_SILU,KC=64>") +
                                f": fused gate/up projection + SiLU*up, M={kern['M']} N={kern['N']} K={kern['K']}"),
                     "bytes_per_launch": kern["bytes"], "ms_per_launch": round(kern["ms"], 5),
                     "measured_stream_read_GBps": round(kern["stream_GBps"], 1),
                     "frac_of_measured_stream": round(achieved / kern["stream_GBps"], 4)},
    }
    if sweep:
        res["sweep"] = sweep
    if cache_sweep:
        res["cache_sweep"] = cache_sweep
    if fused_sweep:
        res["fused_sweep"] = fused_sweep
    if depth_sweep:
        res["depth_sweep"] = depth_sweep
    if training:
        res["training_forward"] = training
    if not args.no_cpu_baseline and param_bytes <= 100e9:
        res["cpu_baseline"] = cpu_baseline(wl, T, n0, weights)
    if not args.only_main and wl.name == "llama7b":
        model.close()
        del model
        torch.cuda.empty_cache()
        # Objects beside the headline: a failure in one of them (say, too little free memory for the 70B model) is
        # recorded in its place and must not take the result line with it.
        def optional(key, fn):
            try:
                res[key] = fn()
            except Exception as exc:                 # noqa: BLE001 - reported, not swallowed
                res[key] = {"error": f"{type(exc).__name__}: {exc}"[:300]}
                torch.cuda.empty_cache()

        if not training:        # the forward pass of the training stage over 2048 tokens, on a model of its own
            def train_object():
                wl_tr = wl.with_(max_cache=2048 + 256)
                m_tr = B.HTModel(B.make_config(wl_tr, max_tree=128), weights, dev)
                try:
                    return time_training_forward(m_tr, 2048)
                finally:
                    m_tr.close()
            optional("training_forward", train_object)
        del weights
        torch.cuda.empty_cache()
        optional("attention_op", lambda: time_attention_op(dev))
        optional("llama13b", lambda: time_second_workload("llama13b", dev, [1, 16, 32, 64, 128], max(5, args.steps),
                                                          also_layers=(25, 30, 35)))
        optional("llama70b", lambda: time_second_workload("llama70b", dev, [1, 64], max(5, args.steps // 3)))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
