"""Counter-based, integer-exact synthetic tensors.

Every element is a pure function of (seed, tensor id, flat element index), computed with
64-bit integer hashing, so the same bits come out on the host and on the GPU, in any chunking,
and a single layer of a 70B-shaped model can be regenerated without generating the rest.

Element recipe (shared by the torch implementation below and the pure-Python reference used
to pin it):

    key   = seed * GOLDEN + tensor_id * TWEAK                       (mod 2^64)
    h_j   = splitmix64_finalizer(key + (3 * idx + j) * GOLDEN),     j = 0, 1, 2
    S     = sum of the twelve 16-bit lanes of h_0, h_1, h_2         (0 .. 12 * 65535)
    z     = (S - 393210) / 65536          # Irwin-Hall(12): mean 0, std 1, |z| <= 6, exact in fp32
    value = fp32(mean) + fp32(sigma) * z  # one fp32 multiply, one fp32 add, then RNE to storage dtype

Token ids use one hash: top 31 bits of splitmix64_finalizer(key + idx * GOLDEN), mod vocab.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence

import torch

_M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
TWEAK = 0xD1B54A32D192ED03
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB


def _s64(u: int) -> int:
    """Two's-complement view of an unsigned 64-bit value as a Python int in int64 range."""
    u &= _M64
    return u - (1 << 64) if u >= (1 << 63) else u


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical shift right on an int64 tensor (torch's >> is arithmetic)."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    z = z ^ _lsr(z, 30)
    z = z * _s64(_C1)
    z = z ^ _lsr(z, 27)
    z = z * _s64(_C2)
    z = z ^ _lsr(z, 31)
    return z


def _key(seed: int, tensor_id: int) -> int:
    return (seed * GOLDEN + tensor_id * TWEAK) & _M64


# ----------------------------------------------------------------------------- pure-Python pin
def _mix_py(z: int) -> int:
    z &= _M64
    z ^= z >> 30
    z = (z * _C1) & _M64
    z ^= z >> 27
    z = (z * _C2) & _M64
    z ^= z >> 31
    return z


def counter_u64_reference(seed: int, tensor_id: int, idx: int) -> int:
    """Lane sum S for one element, in plain Python integers (slow; pins the torch version)."""
    key = _key(seed, tensor_id)
    s = 0
    for j in range(3):
        h = _mix_py(key + (3 * idx + j) * GOLDEN)
        s += (h & 0xFFFF) + ((h >> 16) & 0xFFFF) + ((h >> 32) & 0xFFFF) + (h >> 48)
    return s


def counter_token_reference(seed: int, stream_id: int, idx: int, vocab: int) -> int:
    h = _mix_py(_key(seed, stream_id) + idx * GOLDEN)
    return (h >> 33) % vocab


# ----------------------------------------------------------------------------- torch generators
def _lane_sum(key: int, idx: torch.Tensor) -> torch.Tensor:
    s = torch.zeros_like(idx)
    for j in range(3):
        ctr = (idx * 3 + j) * _s64(GOLDEN) + _s64(key)
        h = _mix(ctr)
        s = s + (h & 0xFFFF) + (_lsr(h, 16) & 0xFFFF) + (_lsr(h, 32) & 0xFFFF) + _lsr(h, 48)
    return s


def counter_normal(seed: int, tensor_id: int, shape: Sequence[int], sigma: float, mean: float = 0.0,
                   device: str | torch.device = "cpu", dtype: torch.dtype = torch.float32,
                   chunk: int = 1 << 24) -> torch.Tensor:
    """Tensor of approximately N(mean, sigma^2) values, bit-identical on every device."""
    numel = 1
    for s in shape:
        numel *= int(s)
    out = torch.empty(numel, device=device, dtype=dtype)
    key = _key(seed, tensor_id)
    sig = torch.tensor(sigma, dtype=torch.float32, device=device)
    mu = torch.tensor(mean, dtype=torch.float32, device=device)
    for start in range(0, numel, chunk):
        end = min(numel, start + chunk)
        idx = torch.arange(start, end, device=device, dtype=torch.int64)
        z = (_lane_sum(key, idx) - 393210).to(torch.float32) / 65536.0
        val = torch.mul(z, sig)
        if mean != 0.0:
            val = torch.add(val, mu)
        out[start:end] = val.to(dtype)
    return out.view(*shape)


def counter_tokens(seed: int, stream_id: int, count: int, vocab: int,
                   device: str | torch.device = "cpu") -> torch.Tensor:
    """`count` token ids in [0, vocab), int32."""
    idx = torch.arange(count, device=device, dtype=torch.int64)
    h = _mix(idx * _s64(GOLDEN) + _s64(_key(seed, stream_id)))
    return (_lsr(h, 33) % vocab).to(torch.int32)


# ----------------------------------------------------------------------------- model weights
TENSOR_IDS = {
    "tok_emb": 1, "final_norm": 2, "lm_head": 3,
    "w_transfer": 50,             # + step index
    "layer_base": 1000,           # + 16 * layer + slot below
    "attn_norm": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "ffn_norm": 5, "w_gate": 6, "w_up": 7, "w_down": 8,
}
PROMPT_STREAM = 7
_LAYER_SLOTS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def _dims(shape):
    d, hq, hkv, hd, f = shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn
    return {
        "attn_norm": (d,), "wq": (hq * hd, d), "wk": (hkv * hd, d), "wv": (hkv * hd, d), "wo": (d, hq * hd),
        "ffn_norm": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }


def layer_weights(shape, seed: int, layer: int, device="cpu", dtype: torch.dtype = torch.float32,
                  sigma: float = 0.02) -> Dict[str, torch.Tensor]:
    """The nine tensors of one decoder layer (same values `make_weights` gives for that layer)."""
    dims = _dims(shape)
    out = {}
    for name in _LAYER_SLOTS:
        tid = TENSOR_IDS["layer_base"] + 16 * layer + TENSOR_IDS[name]
        out[name] = counter_normal(seed, tid, dims[name], sigma, 1.0 if name.endswith("norm") else 0.0,
                                   device=device, dtype=dtype)
    return out


def make_weights(shape, seed: int, device: str | torch.device = "cpu", dtype: torch.dtype = torch.float32,
                 layers: Optional[Iterable[int]] = None, sigma: float = 0.02,
                 with_head: bool = True) -> Dict[str, object]:
    """Random-init weights of a Llama-style decoder plus the k hidden-transfer maps.

    `shape` needs attributes n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, k.
    All matrices are N(0, sigma^2), row-major [out, in]; norm gains are 1 + N(0, sigma^2) so a
    dropped gain multiply is visible.  `layers` restricts generation to a subset of layer indices
    (their matrices are None, their norm gains are still generated) so a single layer of a large
    shape can be rebuilt on the host, or a large model can be supplied to the GPU layer by layer.
    """
    d, v = shape.d_model, shape.vocab

    def gen(tid, shp, is_gain=False):
        return counter_normal(seed, tid, shp, sigma, 1.0 if is_gain else 0.0, device=device, dtype=dtype)

    w: Dict[str, object] = {}
    w["tok_emb"] = gen(TENSOR_IDS["tok_emb"], (v, d))
    w["final_norm"] = gen(TENSOR_IDS["final_norm"], (d,), True)
    w["lm_head"] = gen(TENSOR_IDS["lm_head"], (v, d)) if with_head else None
    w["w_transfer"] = [gen(TENSOR_IDS["w_transfer"] + i, (d, d)) for i in range(shape.k)]
    want = set(range(shape.n_layers)) if layers is None else set(layers)
    for name in _LAYER_SLOTS:
        w[name] = []
    dims = _dims(shape)
    for layer in range(shape.n_layers):
        lw = layer_weights(shape, seed, layer, device, dtype, sigma) if layer in want else None
        for name in _LAYER_SLOTS:
            if lw is not None:
                w[name].append(lw[name])
            elif name.endswith("norm"):                  # the small gain vectors are always generated
                tid = TENSOR_IDS["layer_base"] + 16 * layer + TENSOR_IDS[name]
                w[name].append(gen(tid, dims[name], True))
            else:
                w[name].append(None)
    return w
