"""The packed skinny product for callers that cannot allocate (`ht_skinny_gemm_packed_noalloc`: split-K partial sums
in a device array of the library's own) against `ht_skinny_gemm_packed` with a caller's scratch buffer, through the
C ABI: the same kernels and K split, so the same bits; two calls in a row, the second smaller, so that what the
first left in the shared array cannot leak into the second.  Needs a real MI355X."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from ht_inputs import counter_normal
from oracle import ht_oracle as O

DEV = "cuda:0"


def _case(B, M, N, K, seed):
    Mp = B.ht_padded_rows(M)
    a = torch.zeros(Mp, K, dtype=torch.bfloat16, device=DEV)
    a[:M] = counter_normal(seed, 41, (M, K), 1.0, device=DEV, dtype=torch.bfloat16)
    w = counter_normal(seed, 42, (N, K), 0.05, device=DEV, dtype=torch.bfloat16)
    packed = torch.empty(B.ht_weight_pack_bytes(N, K), dtype=torch.uint8, device=DEV)
    B.ht_weight_pack(w, N, K, packed)
    scratch = torch.empty(B.ht_skinny_gemm_scratch_bytes(M, N, K), dtype=torch.uint8, device=DEV)
    want = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    got = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    return a, w, packed, scratch, want, got


def test_no_alloc_product_equals_the_scratch_argument_product_on_two_calls_in_a_row():
    import paper_2404_12022_amd.binding as B
    # split-K shapes (the partial sums go through the library's array); the second call is smaller in M, N and K
    shapes = [(64, 4096, 11008), (17, 1024, 4096)]
    cases = [_case(B, *shape, seed=50 + i) for i, shape in enumerate(shapes)]
    before = torch.cuda.memory_allocated()
    for (M, N, K), (a, w, packed, scratch, want, got) in zip(shapes, cases):
        print(f"no-alloc product M={M} N={N} K={K}", flush=True)
        B.ht_skinny_gemm_packed_noalloc(a, packed, M, N, K, got)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for (M, N, K), (a, w, packed, scratch, want, got) in zip(shapes, cases):
        B.ht_skinny_gemm_packed(a, packed, M, N, K, want, scratch)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"M={M} N={N} K={K}: differs from the product with a scratch argument"
        exact = O.linear(a[:M].float().cpu().numpy().astype(np.float64), w.float().cpu().numpy().astype(np.float64))
        err = np.max(np.abs(got.cpu().numpy().astype(np.float64) - exact))
        assert err <= 2e-5 * np.sqrt(K) * float(a[:M].float().abs().max()) * 0.05 * 8 + 1e-6, err


def test_no_alloc_product_without_a_split_and_beyond_the_array():
    import paper_2404_12022_amd.binding as B
    M, N, K = 16, 32000, 256                       # vocabulary-sized N: never split, the array is not touched
    a, w, packed, scratch, want, got = _case(B, M, N, K, seed=60)
    B.ht_skinny_gemm_packed_noalloc(a, packed, M, N, K, got)
    B.ht_skinny_gemm_packed(a, packed, M, N, K, want, scratch)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
    # 8 splits x 128 rows x 4352 columns of fp32 partial sums are 17 MiB: more than the library's 16 MiB
    M, N, K = 128, 4352, 16384
    assert 8 * M * N * 4 > B.HT_NOALLOC_SCRATCH_BYTES
    a = torch.zeros(128, K, dtype=torch.bfloat16, device=DEV)
    packed = torch.zeros(B.ht_weight_pack_bytes(N, K), dtype=torch.uint8, device=DEV)
    out = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    with pytest.raises(B.HTError) as e:
        B.ht_skinny_gemm_packed_noalloc(a, packed, M, N, K, out)
    assert e.value.code == B.HT_ECAPACITY
    with pytest.raises(B.HTError) as e:
        B.ht_skinny_gemm_packed_noalloc(a, packed, 0, N, K, out)
    assert e.value.code == B.HT_EINVAL
