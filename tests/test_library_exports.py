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
    assert sorted(probe.EXPORTS) == syms and len(syms) == 5
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
    assert lib.etv_status_string(-5) == b"not implemented"
    # a replica of a contiguous cache is a defined operation that is not built: refused on the host, before any pointer is used
    cd = api.CacheDesc(B=1, Hkv=2, d=64, elem_bytes=2, n_layers=1, block_size=0, max_blocks=0, num_blocks=0, P_cap=64,
                       reserved=0, cache_layer_stride=64 * 2 * 64)
    assert lib.etv_replicate_branches(ctypes.byref(cd), None, None, None, None, None, 1, None, 0, None, None, None, None,
                                      None) == -5
    dsc = api.AttnDesc(B=1, T_max=60, Hq=32, Hkv=8, d=128, dtype=api.BF16, block_size=0, max_blocks=0, num_blocks=0,
                       P_cap=2100, P_max=2048, scale=0.0, kv_split=0, flags=0)
    ws = api.tree_verify_attention_workspace_bytes(dsc)
    assert ws >= 256
    dsc.kv_split = 64
    assert api.tree_verify_attention_workspace_bytes(dsc) >= 1 * 32 * 60 * 32 * 130 * 4
    assert api.evaluate_posterior_workspace_bytes(1, 60, 32000) == 60 * 8 * 8


def test_launch_plan_is_reported_and_follows_the_tuning_flags():
    """Host-only: the plan call shows what the cost model picks, and kv_split / the flags override it."""
    def desc(B, T, P, paged, **kw):
        return api.AttnDesc(B=B, T_max=T, Hq=32, Hkv=8, d=128, dtype=api.BF16, block_size=16 if paged else 0,
                            max_blocks=(P + T + 15) // 16 + 1, num_blocks=0, P_cap=P + T, P_max=P, scale=0.0,
                            kv_split=kw.get("kv_split", 0), flags=kw.get("flags", 0))
    big = api.tree_verify_attention_plan(desc(32, 128, 4096, True))
    assert big["mfma"] == 1 and big["n_splits"] == 1 and big["kv_split"] == 4096 and big["workgroups"] == 32 * 8 * big["row_groups"]
    assert big["wavefronts"] * (1 if not big["key_halves"] else 0.5) * big["row_groups"] >= 16      # 16 chunks of 32 rows
    c2 = api.tree_verify_attention_plan(desc(1, 60, 2048, False))
    assert c2["n_splits"] > 1 and c2["kv_split"] % 64 == 0 and c2["kv_split"] * c2["n_splits"] >= 2048
    forced = api.tree_verify_attention_plan(desc(1, 60, 2048, False, kv_split=512, flags=api.ATTN_FLAG_WHOLE_TILE | api.ATTN_FLAG_SMALL_WG))
    assert forced["kv_split"] == 512 and forced["n_splits"] == 4 and forced["key_halves"] == 0 and forced["wavefronts"] == 4
    large = api.tree_verify_attention_plan(desc(1, 60, 2048, False, flags=api.ATTN_FLAG_LARGE_WG | api.ATTN_FLAG_WHOLE_TILE))
    assert large["wavefronts"] == 8 and large["key_halves"] == 0
    # split slots follow the sequences' lengths for batches of 2 .. 64 sequences, unless the flag keeps one split size
    assert big["balanced_splits"] == 0 and c2["balanced_splits"] == 0             # no splits / one sequence
    ragged = api.tree_verify_attention_plan(desc(8, 60, 8192, True))
    assert ragged["n_splits"] > 1 and ragged["balanced_splits"] == 1
    assert ragged["workgroups"] == 8 * ragged["n_splits"] * 8 * ragged["row_groups"]
    kept = api.tree_verify_attention_plan(desc(8, 60, 8192, True, flags=api.ATTN_FLAG_UNIFORM_SPLITS))
    assert kept["balanced_splits"] == 0 and kept["n_splits"] == ragged["n_splits"]
    assert api.tree_verify_attention_plan(desc(65, 12, 8192, True, kv_split=1024))["balanced_splits"] == 0
    ws = api.tree_verify_attention_workspace_bytes(desc(8, 60, 8192, True))
    assert ws >= 8 * ragged["n_splits"] * 32 * 60 * 130 * 4 + 64 * 8                  # partials + the split table
    f32 = api.AttnDesc(B=1, T_max=15, Hq=4, Hkv=4, d=64, dtype=api.F32, block_size=0, max_blocks=0, num_blocks=0,
                       P_cap=200, P_max=128, scale=0.0, kv_split=0, flags=0)
    assert api.tree_verify_attention_plan(f32)["mfma"] == 0


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(api.AttnDesc) == 14 * 4
    assert ctypes.sizeof(api.AttnPlan) == 8 * 4 + 8
    assert ctypes.sizeof(api.CommitDesc) == 12 * 4 + 8
