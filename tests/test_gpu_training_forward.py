"""Forward pass of the training stage with its distillation loss (`ht_training_forward`, Sec. 3.3), HIP path against
the oracle, through the C ABI.  Needs a real MI355X.

Float stages (logits of the hidden states and of the pseudo states) are compared with the fp64 oracle at the model's
tolerance; the KL terms are compared with the oracle's formula applied to the GPU's own logits (<= 2e-5 + 1e-5 |KL|:
the kernel works in float32, three sums over the vocabulary and a difference of two logarithms whose size grows with
the spread of the logits) and, on fp32 models, with the oracle's own terms.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from ht_inputs import WORKLOADS, make_weights
from oracle import ht_oracle as O
from helpers import oracle_model, prompt_of, tree_of

DEV = "cuda:0"


def _B():
    import paper_2404_12022_amd.binding as B
    return B


def _H():
    import gpu_harness as H
    return H


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("rows,V", [(4, 32000), (3, 1001), (6, 40), (2, 4099)])
def test_kl_rows_match_the_definition(rows, V):
    B = _B()
    gen = torch.Generator().manual_seed(V)
    z = (torch.randn(2 * rows + 2, V, generator=gen) * 2.5).float()
    z[1] = z[rows + 2]                                           # one pair of identical rows: exactly zero
    zn = z.numpy().astype(np.float64)
    kl = torch.full((rows,), -1.0, dtype=torch.float32, device=DEV)
    B.ht_kl_divergence_rows(z.to(DEV), 1, rows + 2, rows, kl)
    torch.cuda.synchronize()
    got = kl.cpu().numpy().astype(np.float64)
    want = np.array([O.kl_divergence(zn[1 + p], zn[rows + 2 + p]) for p in range(rows)])
    say(f"kl rows V={V}: max-abs error {np.max(np.abs(got - want)):.2e}, values {want[1]:.3f}..")
    assert np.all(np.abs(got - want) <= 2e-5 + 1e-5 * np.abs(want)) and abs(got[0]) <= 1e-6


def _compare(wl, tensors_gpu, tensors_cpu, n, step, max_tree, exact, batched=False):
    B, H = _B(), _H()
    model = oracle_model(wl, tensors_cpu)
    toks = prompt_of(wl, n)
    res = O.training_forward(model, toks, step)
    gpu = H.gpu_model(wl, tensors_gpu, max_tree=max_tree)
    z = torch.zeros(n, wl.vocab, dtype=torch.float32, device=DEV)
    zp = torch.zeros(n - step + 1, wl.vocab, dtype=torch.float32, device=DEV)
    if batched:
        kl, loss = gpu.ht_training_forward_batched(step, toks, z, zp)
    else:
        kl, loss = gpu.ht_training_forward(step, toks, z, zp)
    torch.cuda.synchronize()
    assert batched or gpu.ht_cache_len() == n
    zc, zpc = H.cpu(z), H.cpu(zp)
    e1 = H.assert_close(zc, res["Z"], wl.dtype, "logits of the hidden states")
    e2 = H.assert_close(zpc, res["Zp"][:n - step + 1], wl.dtype, "logits of the pseudo states")
    assert len(kl) == n - step - 1 == len(res["kl"])
    own = np.array([O.kl_divergence(zpc[j], zc[j + step]) for j in range(n - step - 1)])
    err_own = float(np.max(np.abs(np.array(kl) - own))) if len(kl) else 0.0
    assert np.all(np.abs(np.array(kl) - own) <= 2e-5 + 1e-5 * np.abs(own)), \
        f"KL terms off the definition on the GPU's own logits by {err_own:.2e} (largest term {np.max(own):.3f})"
    assert abs(loss - float(np.sum(np.array(kl, dtype=np.float64)))) <= 1e-9 * max(1.0, abs(loss))
    if exact:
        err = float(np.max(np.abs(np.array(kl) - res["kl"]))) if len(kl) else 0.0
        assert err <= 2e-5 + 1e-3 * float(np.max(res["kl"])), f"KL terms differ from the oracle's by {err:.2e}"
        assert abs(loss - res["loss"]) <= 2e-5 * len(kl) + 1e-3 * res["loss"]
    say(f"  {wl.name} n={n} step={step} rows/pass<={max_tree}: logits {e1:.2e} / {e2:.2e}, KL vs definition {err_own:.2e} "
        f"(largest term {float(np.max(own)) if len(own) else 0.0:.3f}), "
        f"loss {loss:.6f} (oracle {res['loss']:.6f})")
    gpu.close()


@pytest.mark.parametrize("name,n,max_tree", [("tiny", 40, 16), ("tiny", 63, 128), ("tiny_k3", 29, 9), ("tiny_t123", 50, 32),
                                             ("tiny_t112", 23, 128), ("tiny", 5, 16)])
def test_tiny_fp32_training_forward_every_step(name, n, max_tree):
    wl = WORKLOADS[name]
    say(f"training forward {name}")
    for step in range(1, wl.k + 1):
        _compare(wl, None, None, n, step, max_tree, exact=True)


def test_shortest_sequences_and_chunk_tails():
    """n = step + 2 (a single loss term), chunks of one position (max_tree = step + 2), and tails shorter than the
    lookahead."""
    wl = WORKLOADS["tiny_k3"]
    for step in (1, 2, 3):
        _compare(wl, None, None, step + 2, step, 16, exact=True)
        _compare(wl, None, None, 9, step, step + 2, exact=True)
        _compare(wl, None, None, 15, step, 2 * 7 + step, exact=True)      # 7 positions per pass: 15 = 7 + 7 + 1


@pytest.mark.parametrize("name", ["tiny_bf16", "tiny_t123_bf16"])
def test_tiny_bf16_training_forward(name):
    wl = WORKLOADS[name]
    say(f"training forward {name}")
    for step in range(1, wl.k + 1):
        _compare(wl, None, None, 45, step, 24, exact=False)


def test_llama7b_width_two_layers_training_forward():
    """Full 7B widths and vocabulary, 2 layers, 150 tokens in chunks of 62 or 63 positions (128-row passes)."""
    H = _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), max_cache=512)
    say("7B-width 2 layers, training forward: generating weights")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    for step in (1, 3):
        _compare(wl, tensors, cpu_tensors, 150, step, 128, exact=False)


def test_training_forward_state_and_error_codes():
    B, H = _B(), _H()
    wl = WORKLOADS["tiny"].with_(max_cache=64)
    parent, rank = tree_of(wl)
    gpu = H.gpu_model(wl, max_tree=16)
    gpu.ht_set_tree(parent, rank)
    toks = prompt_of(wl, 20)
    for step, n, code in ((0, 20, B.HT_EINVAL), (3, 20, B.HT_EINVAL), (1, 2, B.HT_EINVAL), (2, 3, B.HT_EINVAL),
                          (1, 58, B.HT_ECAPACITY)):
        with pytest.raises(B.HTError) as e:
            gpu.ht_training_forward(step, prompt_of(wl, n))
        assert e.value.code == code, (step, n)
    with pytest.raises(B.HTError) as e:
        gpu.ht_training_forward(1, toks[:5] + [wl.vocab] + toks[6:])
    assert e.value.code == B.HT_EINVAL
    kl, loss = gpu.ht_training_forward(1, toks)
    assert len(kl) == 18 and all(v > 0 for v in kl) and abs(loss - sum(kl)) < 1e-6
    again = gpu.ht_training_forward(1, toks)
    assert again == (kl, loss)                                       # same kernels, same values
    with pytest.raises(B.HTError) as e:                              # the cache holds the sequence but no pending root
        gpu.ht_tree_verify_step(None, None, None)
    assert e.value.code == B.HT_ESTATE
    gpu.ht_prefill(toks)                                             # decoding goes on with the tree set before
    out = []
    for _ in range(4):
        gpu.ht_transfer(None, None)
        gpu.ht_tree_verify_step(None, None, None)
        out += gpu.ht_accept_and_compact()[1]
    assert out == oracle_model(wl).ar_greedy(toks, len(out))
    gpu.close()


@pytest.mark.parametrize("seed", [f"any{i}" for i in range(6)] + [f"packed{i}" for i in range(6)])
def test_random_model_shapes_training_forward(seed):
    """The random shapes of the decoding suite (grouped heads, odd widths and vocabularies, several transfer layers,
    both kernel families), every transfer step, a random sequence length and rows per pass."""
    from test_gpu_parity import _random_shape, _random_packed_shape
    wl, _, _ = _random_shape(int(seed[3:])) if seed.startswith("any") else _random_packed_shape(int(seed[6:]))
    rng = np.random.default_rng(int(seed[-1]) + 17)
    n = int(rng.integers(wl.k + 2, 90))
    max_tree = int(rng.integers(wl.k + 2, 129))
    wl = wl.with_(max_cache=(n + 64 + 7) // 8 * 8)
    say(f"training forward, random shape {seed}: {wl.dtype} layers={wl.n_layers} d={wl.d_model} heads={wl.n_heads}/"
        f"{wl.n_kv_heads}x{wl.head_dim} vocab={wl.vocab} k={wl.k} t={wl.transfer_layers} n={n} rows/pass<={max_tree}")
    for step in range(1, wl.k + 1):
        _compare(wl, None, None, n, step, max_tree, exact=wl.dtype == "f32")


# ------------------------------------------------------------------ all positions in one pass per block
def _packed_small(**kw):
    from helpers import small_workload
    base = dict(name="batched", n_layers=3, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64, d_ffn=272, vocab=512, k=3,
                transfer_layers=(1, 2, 2), dtype="bf16", prompt_len=8, max_cache=1024, tree_size=8, branching=(2, 2, 1),
                seed=5151)
    base.update(kw)
    return small_workload(**base)


@pytest.mark.parametrize("n", [5, 77, 128, 129, 300, 515])
def test_batched_training_forward_small_model(n):
    """Sequence lengths below, at and above the 128-row attention chunks and the 128-token product tiles, with one, two
    and several pseudo-row passes, the last one short; every transfer step (joins at two different layers)."""
    wl = _packed_small()
    say(f"batched training forward, small packed model, n = {n}")
    for step in (1, 2, 3):
        if n >= step + 2:
            _compare(wl, None, None, n, step, 64, exact=False, batched=True)


def test_batched_training_forward_wide_heads_and_grouped_queries():
    wl = _packed_small(name="batched128", d_model=256, n_heads=4, n_kv_heads=1, head_dim=128, d_ffn=400, vocab=1008, k=2,
                       transfer_layers=(1, 1), n_layers=2)
    say("batched training forward, 128-wide heads, four query heads on one key/value head")
    for step in (1, 2):
        _compare(wl, None, None, 260, step, 64, exact=False, batched=True)


def test_batched_training_forward_llama7b_width_and_both_paths_agree():
    """Full 7B widths and vocabulary, 2 layers, 300 tokens: against the oracle, and the loss against the chunked
    `ht_training_forward` on the same model (two bf16 computations of the same sums)."""
    B, H = _B(), _H()
    wl = WORKLOADS["llama7b"].with_(n_layers=2, transfer_layers=(1, 1, 1), max_cache=640)
    say("7B-width 2 layers, batched training forward: generating weights")
    tensors = make_weights(wl, wl.seed, H.DEV, torch.bfloat16)
    cpu_tensors = {k: ([t.cpu() for t in v] if isinstance(v, list) else v.cpu()) for k, v in tensors.items()}
    _compare(wl, tensors, cpu_tensors, 300, 2, 128, exact=False, batched=True)
    gpu = H.gpu_model(wl, tensors, max_tree=128)
    toks = prompt_of(wl, 300)
    kl_a, loss_a = gpu.ht_training_forward(2, toks)
    kl_b, loss_b = gpu.ht_training_forward_batched(2, toks)
    say(f"  loss chunked {loss_a:.6f}, batched {loss_b:.6f}")
    assert abs(loss_a - loss_b) <= 0.03 * abs(loss_a)
    with pytest.raises(B.HTError) as e:                              # the cache holds nothing usable afterwards
        gpu.ht_tree_verify_step(None, None, None)
    assert e.value.code == B.HT_ESTATE
    gpu.close()


def test_batched_training_forward_error_codes():
    B, H = _B(), _H()
    f32 = H.gpu_model(WORKLOADS["tiny"], max_tree=16)
    with pytest.raises(B.HTError) as e:
        f32.ht_training_forward_batched(1, prompt_of(WORKLOADS["tiny"], 20))
    assert e.value.code == B.HT_EUNSUPPORTED                         # fp32 models have no packed weights
    f32.close()
    wl = _packed_small(max_cache=320)
    gpu = H.gpu_model(wl, max_tree=16)
    for step, n, code in ((0, 20, B.HT_EINVAL), (4, 20, B.HT_EINVAL), (2, 3, B.HT_EINVAL), (1, 321, B.HT_ECAPACITY)):
        with pytest.raises(B.HTError) as e:
            gpu.ht_training_forward_batched(step, prompt_of(wl, n))
        assert e.value.code == code, (step, n)
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.HTError) as e:
        gpu.ht_training_forward_batched(1, prompt_of(wl, 20), workspace=small)
    assert e.value.code == B.HT_EINVAL
    kl, loss = gpu.ht_training_forward_batched(1, prompt_of(wl, 20))
    assert len(kl) == 18 and abs(loss - sum(kl)) < 1e-5
    gpu.close()
