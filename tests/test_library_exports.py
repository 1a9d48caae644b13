"""CPU-side checks of the boundary: the built library loads and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_2603_08088_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header="eagletv.h", prefix="etv_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_binding_lists_them_all():
    syms = _declared_symbols()
    assert len(syms) >= 10
    assert os.path.exists(api.LIB_PATH), "build the library first: python -m paper_2603_08088_amd.build"
    lib = ctypes.CDLL(api.LIB_PATH)
    for s in syms:
        assert hasattr(lib, s), s
    assert sorted(api.EXPORTS) == syms


def test_probe_library_exports_its_header_and_the_product_library_holds_no_probe():
    from paper_2603_08088_amd import probe
    syms = _declared_symbols("eagletv_probe.h", "etvp_")
    assert sorted(probe.EXPORTS) == syms and len(syms) == 3
    lib = ctypes.CDLL(probe.LIB_PATH)
    for s in syms:
        assert hasattr(lib, s), s
    assert probe.mfma_bf16_probe_flops(1) == 2048 * 4 * 16 * 2 * 32 * 32 * 16
    product = ctypes.CDLL(api.LIB_PATH)
    assert not hasattr(product, "etv_hbm_read_probe") and not hasattr(product, "etvp_hbm_read_probe")


def test_host_only_calls_need_no_gpu():
    lib = api.lib()
    assert b"gfx950" in lib.etv_version()
    assert lib.etv_status_string(0) == b"ok" and lib.etv_status_string(-3) == b"workspace too small"
    dsc = api.AttnDesc(B=1, T_max=60, Hq=32, Hkv=8, d=128, dtype=api.BF16, block_size=0, max_blocks=0, num_blocks=0,
                       P_cap=2100, P_max=2048, scale=0.0, kv_split=0, flags=0)
    ws = api.tree_verify_attention_workspace_bytes(dsc)
    assert ws >= 256
    dsc.kv_split = 64
    assert api.tree_verify_attention_workspace_bytes(dsc) >= 1 * 32 * 60 * 32 * 130 * 4
    assert api.evaluate_posterior_workspace_bytes(1, 60, 32000) == 60 * 8 * 8


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(api.AttnDesc) == 14 * 4
    assert ctypes.sizeof(api.CommitDesc) == 12 * 4 + 8
