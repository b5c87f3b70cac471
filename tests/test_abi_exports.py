"""CPU-only: the C-ABI library loads and exports every entry point include/ht.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2404_12022_amd", "libht.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ht.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ht_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_named_entry_points():
    names = declared_symbols()
    for must in ("ht_init_model", "ht_transfer", "ht_tree_verify_step", "ht_accept_and_compact"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} is declared in ht.h but not exported by libht.so"


def test_binding_names_match_the_header():
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    import paper_2404_12022_amd.binding as B
    assert sorted(B.EXPORTS) == declared_symbols()
    # host-only argument checks: no GPU is touched before validation fails
    cfg = B.ht_config()
    out = ctypes.c_size_t(0)
    assert B.lib.ht_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)) == B.HT_EINVAL
    assert b"dimension" in B.lib.ht_last_error()
    assert B.lib.ht_padded_rows(1) == 16 and B.lib.ht_padded_rows(64) == 64 and B.lib.ht_padded_rows(65) == 128
    from ht_inputs import WORKLOADS
    good = B.make_config(WORKLOADS["llama7b"])
    assert B.ht_workspace_bytes(good) > 32 * 2 * 1024 * 4096 * 2          # at least the KV cache
    good.transfer_layer[1] = 25                                            # 24, 25, 24: layers may not decrease
    assert B.lib.ht_workspace_bytes(ctypes.byref(good), ctypes.byref(out)) == B.HT_EINVAL
    good.transfer_layer[2] = 30                                            # 24, 25, 30 is fine
    assert B.lib.ht_workspace_bytes(ctypes.byref(good), ctypes.byref(out)) == B.HT_OK


def test_binding_constants_match_the_header():
    """Limits and codes the binding re-types (it cannot include a C header) against include/ht.h."""
    if not os.path.exists(LIB):
        pytest.skip("library not built")
    import paper_2404_12022_amd.binding as B
    text = open(os.path.join(ROOT, "include", "ht.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    enums = dict((k, int(v)) for k, v in re.findall(r"\b(HT_[A-Z_0-9]+)\s*=\s*(-?\d+)", text))
    for name in ("HT_OK", "HT_EINVAL", "HT_ECAPACITY", "HT_ETREE", "HT_ESTATE", "HT_EHIP", "HT_EUNSUPPORTED", "HT_F32", "HT_BF16",
                 "HT_MAX_TRANSFER", "HT_MAX_TREE", "HT_MAX_ROWS", "HT_MAX_TOPK", "HT_MAX_LOOP_STEPS", "HT_BUF_DRAFT_LOGITS",
                 "HT_BUF_K_CACHE", "HT_BUF_V_CACHE", "HT_BUF_FUSED_DRAFT_LOGITS", "HT_BUF_TREE_PARENT", "HT_BUF_TREE_RANK"):
        assert getattr(B, name) == enums[name], name
    m = re.search(r"#define\s+HT_NOALLOC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert B.HT_NOALLOC_SCRATCH_BYTES == int(m.group(1)) << int(m.group(2))
    assert B.lib.ht_padded_rows(129) == 256 and B.lib.ht_padded_rows(256) == 256


def test_bench_refuses_more_than_one_gpu():
    """One GPU is the whole target: `bench.py --gpus N` with N > 1 exits with a message and prints no result line."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and not r.stdout.strip()
