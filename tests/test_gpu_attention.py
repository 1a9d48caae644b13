"""GPU parity of tree_verify_attention against the fp64 oracle.

Tolerances (max-abs over all valid output elements): 1e-5 for fp32 inputs, 2e-2 for bf16 inputs with
fp32 accumulation.  Because outputs of flat softmaxes are small (std about sqrt(e/P)), every case also
bounds the scaled error |gpu - ref| / (|ref| + rms(ref)) by 1e-5 (fp32) / 2e-2 (bf16; bf16 rounding of the probabilities and of
the output alone is 2^-9 relative), and "peaked" twins (Q x 4) make the outputs O(1).
"""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import api, synth
from gpu_helpers import DevWorkload, attention_errors, gpu_attention, to_dev, to_host_f64, bits_of
from helpers import random_tree

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
REL_TOL = {"f32": 1e-5, "bf16": 2e-2}   # max of |err| / (|ref| + rms(ref))

# worst observed errors per test, written as JSON to $ETV_ERROR_REPORT when that is set (a record for the
# record of the tolerances actually needed; the assertions do not depend on it)
_WORST = {}


def _record(tag, err, rel):
    name = os.environ.get("PYTEST_CURRENT_TEST", "?").split("::")[-1].split(" ")[0]
    w = _WORST.setdefault(name, {"max_abs": 0.0, "scaled": 0.0, "worst_case": ""})
    w["max_abs"] = max(w["max_abs"], err)
    if rel > w["scaled"]:
        w["scaled"], w["worst_case"] = rel, tag


@pytest.fixture(scope="module", autouse=True)
def _error_report():
    yield
    path = os.environ.get("ETV_ERROR_REPORT")
    if path:
        with open(path, "w") as f:
            json.dump(_WORST, f, indent=1, sort_keys=True)


def _check(wl, *, kv_split=0, flags=0, check_lse=True, rows=None):
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    out, lse = gpu_attention(d, m["bitmask"], kv_split=kv_split, flags=flags)
    torch.cuda.synchronize()
    ref_mask = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    assert np.array_equal(bits_of(m["bitmask"]).view(np.uint64), ref_mask["bitmask"])
    ref, ref_lse = oracle.tree_verify_attention(wl.q, wl.k_cache, wl.v_cache, wl.prefix_len, wl.kt, wl.vt,
                                                ref_mask["dense"], wl.n_nodes, dtype=wl.dtype,
                                                block_table=wl.block_table)
    err, rel, padded_zero = attention_errors(out, ref, wl.n_nodes)
    assert padded_zero, "padded rows must be exact zeros"
    _record(f"{wl.name} B={wl.B} T={wl.T_max} G={wl.Hq // wl.Hkv} P={wl.prefix_len.tolist()[:4]} kv_split={kv_split} flags={flags}",
            err, rel)
    assert err <= TOL[wl.dtype], (wl.name, err)
    assert rel <= REL_TOL[wl.dtype], (wl.name, rel)
    if check_lse:
        g = to_host_f64(lse)
        for b in range(wl.B):
            n = int(wl.n_nodes[b])
            assert np.all(np.isneginf(g[b, :, n:]))
            if n:
                assert np.abs(g[b, :, :n] - ref_lse[b, :, :n]).max() <= (1e-4 if wl.dtype == "f32" else 2e-2)
    return err, rel


def _small(rng, B, T, Hq, Hkv, d, P, dtype, paged, n_nodes=None, q_scale=1.0):
    parents = [random_tree(rng, (n_nodes[b] if n_nodes else T)) for b in range(B)]
    return synth.assemble("small", rng, parents, P, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype, V=512, W=T, paged=paged,
                          T_max=T, with_logits=False, q_scale=q_scale, spare_blocks=3)


def test_config1_tiny_fp32():
    for peaked in (1.0, 4.0):
        rng_wl = synth.config1(with_logits=False, q_scale=peaked)
        _check(rng_wl)
        _check(rng_wl, kv_split=64)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 64)])
@pytest.mark.parametrize("paged", [False, True])
def test_generic_kernel_shapes(dtype, d, paged):
    rng = np.random.default_rng(500 + d)
    # ragged batch, padded node rows, empty prefix, several tiles + ragged tail, G in {1,2,4}
    for (Hq, Hkv, T, P, n) in [(4, 4, 15, [128, 0, 77], [15, 9, 1]), (8, 2, 70, [200, 33], [70, 64]),
                                (4, 2, 128, [130], [128]), (4, 2, 200, [70], [193])]:
        wl = _small(rng, len(P), T, Hq, Hkv, d, P, dtype, paged, n_nodes=n)
        _check(wl)
        _check(wl, kv_split=64)


@pytest.mark.parametrize("T", [1, 8, 16, 31, 32, 33, 60, 64, 65, 96, 127, 128, 129, 160, 192, 193, 255, 256])
def test_mfma_kernel_tree_sizes(T):
    rng = np.random.default_rng(600 + T)
    wl = _small(rng, 2, T, 8, 2, 128, [300, 64], "bf16", False, n_nodes=[T, max(1, T - 3)])
    _check(wl)                    # library-chosen split
    _check(wl, kv_split=64)       # one tile per split
    _check(wl, kv_split=4096)     # single split: direct epilogue
    ref = _check(wl, flags=api.ATTN_FLAG_GENERIC)   # same inputs through the fp32-VALU kernel


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("G,Hkv", [(1, 4), (2, 2), (4, 2), (8, 1)])
def test_mfma_kernel_grouping_ragged_and_edge_prefixes(paged, G, Hkv):
    rng = np.random.default_rng(700 + G)
    P = [0, 1, 63, 64, 65, 500]
    n = [40, 1, 40, 17, 40, 33]
    wl = _small(rng, len(P), 40, G * Hkv, Hkv, 128, P, "bf16", paged, n_nodes=n)
    _check(wl)
    _check(wl, kv_split=128)
    wl4 = _small(rng, 2, 40, G * Hkv, Hkv, 128, [257, 31], "bf16", paged, q_scale=4.0)   # peaked softmax
    _check(wl4)
    _check(wl4, kv_split=64)


@pytest.mark.parametrize("flags", [api.ATTN_FLAG_KEY_HALVES, api.ATTN_FLAG_WHOLE_TILE,
                                   api.ATTN_FLAG_KEY_HALVES | api.ATTN_FLAG_SMALL_WG])
@pytest.mark.parametrize("paged", [False, True])
def test_mfma_kernel_key_halves_and_whole_tiles_agree_with_the_oracle(flags, paged):
    """Both ways of sharing a tile among wavefronts (two wavefronts per 32-row chunk, each with half of the
    tile's keys and a merge at the end; or one wavefront per chunk) on trees from 1 node up, ragged node
    counts, prefixes around the 32- and 64-key boundaries, several tiles, flat and peaked softmaxes."""
    rng = np.random.default_rng(1700 + flags + 100 * paged)
    for T in (1, 3, 8, 9, 16, 24, 32, 40, 64):
        wl = _small(rng, 2, T, 8, 2, 128, [300, 77], "bf16", paged, n_nodes=[T, max(1, T // 2)])
        _check(wl, flags=flags)
        _check(wl, kv_split=64, flags=flags)
    P = [0, 1, 31, 32, 33, 63, 64, 65, 95, 96, 97, 500]
    wl = _small(rng, len(P), 16, 8, 2, 128, P, "bf16", paged, n_nodes=[16, 1, 7, 16, 9, 16, 2, 16, 16, 5, 16, 11])
    _check(wl, flags=flags)
    _check(wl, kv_split=128, flags=flags)
    for G, Hkv in ((1, 4), (8, 1)):
        wl = _small(rng, 2, 12, G * Hkv, Hkv, 128, [700, 130], "bf16", paged, q_scale=4.0)
        _check(wl, flags=flags)
        _check(wl, kv_split=192, flags=flags)
    wl = _small(rng, 2, 32, 8, 2, 128, [3000, 1537], "bf16", paged, q_scale=12.0)   # long, very peaked: many rescales
    _check(wl, kv_split=4096, flags=flags)
    _check(wl, kv_split=1024, flags=flags)


def test_key_halves_merge_is_deterministic():
    """The merge of the two key halves has a fixed order: two launches on the same inputs give the same bits."""
    rng = np.random.default_rng(1800)
    wl = _small(rng, 3, 16, 8, 2, 128, [300, 77, 640], "bf16", True, n_nodes=[16, 5, 16])
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    out, lse = gpu_attention(d, m["bitmask"], kv_split=128, flags=api.ATTN_FLAG_KEY_HALVES)
    out2, lse2 = gpu_attention(d, m["bitmask"], kv_split=128, flags=api.ATTN_FLAG_KEY_HALVES)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(lse, lse2)   # run-to-run deterministic


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(3, 3), (6, 2), (9, 3), (10, 5), (12, 2), (7, 1), (20, 4)])
def test_mfma_kernel_odd_head_counts(paged, Hq, Hkv):
    """Group sizes that are not powers of two (rows of a KV head are packed as node * G + head, so chunks of 32
    straddle nodes and heads) and KV head counts that are not multiples of the XCD count."""
    rng = np.random.default_rng(1900 + Hq * 10 + Hkv)
    for T, P, n in ((11, [130, 64], [11, 5]), (60, [300, 77], [60, 33]), (128, [200], [100])):
        wl = _small(rng, len(P), T, Hq, Hkv, 128, P, "bf16", paged, n_nodes=n)
        _check(wl)
        _check(wl, kv_split=128)
        _check(wl, flags=api.ATTN_FLAG_KEY_HALVES)
        _check(wl, flags=api.ATTN_FLAG_WHOLE_TILE, kv_split=64)


def test_long_prefix_and_many_sequences():
    """A 40k-key prefix (hundreds of tiles per split, many splits) and a batch of 200 one-tile sequences."""
    rng = np.random.default_rng(1950)
    wl = _small(rng, 1, 24, 8, 2, 128, [40000], "bf16", True, q_scale=4.0)
    _check(wl)
    _check(wl, kv_split=40000)      # one split of 625 tiles
    B = 200
    P = [int(x) for x in rng.integers(0, 70, size=B)]
    n = [int(x) for x in rng.integers(0, 13, size=B)]
    wl = _small(rng, B, 12, 4, 2, 128, P, "bf16", True, n_nodes=[max(0, x) for x in n])
    _check(wl)


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("B,T,kv_split", [(2, 40, 64), (7, 60, 256), (8, 200, 128), (64, 12, 64), (65, 12, 64)])
def test_splits_shared_out_by_length_agree_with_the_oracle(paged, B, T, kv_split):
    """Ragged batches with splits: up to 64 sequences the launch's split slots follow the sequences' lengths (every
    sequence cuts its own prefix evenly over its share); the uniform split size is kept beyond 64 sequences and on
    request.  Both against the oracle, with empty prefixes, empty trees and prefixes of a few keys in the batch."""
    rng = np.random.default_rng(4200 + B + T)
    hi = 2000 if B <= 8 else 300
    P = [int(x) for x in rng.integers(0, hi + 1, size=B)]
    n = [int(x) for x in rng.integers(1, T + 1, size=B)]
    P[0], n[0] = hi, T           # the longest sequence sizes the launch
    P[1] = 0                     # no prefix at all
    if B > 2:
        P[2], n[2] = 0, 0        # nothing at all
        P[3], n[3] = 65, 0       # a prefix but no tree
        P[-1] = 3
    wl = _small(rng, B, T, 8, 2, 128, P, "bf16", paged, n_nodes=n, q_scale=2.0)
    d = DevWorkload(wl)

    def desc(flags):
        return api.attn_desc(d.q, d.kt, d.k_cache, d.block_table, d.P_max, kv_split=kv_split, flags=flags)
    plan = api.tree_verify_attention_plan(desc(0))
    assert plan["n_splits"] > 1 and plan["balanced_splits"] == (1 if B <= 64 else 0)
    uniform = api.tree_verify_attention_plan(desc(api.ATTN_FLAG_UNIFORM_SPLITS))
    assert uniform["balanced_splits"] == 0 and uniform["n_splits"] == plan["n_splits"]
    _check(wl, kv_split=kv_split)
    _check(wl, kv_split=kv_split, flags=api.ATTN_FLAG_UNIFORM_SPLITS)


def test_no_leak_from_hidden_tree_rows_padding_and_stale_cache_bf16():
    rng = np.random.default_rng(800)
    wl = _small(rng, 1, 48, 8, 2, 128, [100], "bf16", False, n_nodes=[37])
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    out0, lse0 = gpu_attention(d, m["bitmask"])
    dense = oracle.build_tree_mask(wl.parent, wl.n_nodes)["dense"][0, 0]
    k = 30
    hidden = [j for j in range(48) if not dense[k, j]]
    big = synth.f32_to_bf16_bits(np.full(1, 1e4, dtype=np.float32))[0]
    wl.kt[0, hidden] = big; wl.vt[0, hidden] = big
    wl.k_cache[0, 100:] = big; wl.v_cache[0, 100:] = big
    wl.q[0, 37:] = big
    d2 = DevWorkload(wl)
    out1, lse1 = gpu_attention(d2, m["bitmask"])
    torch.cuda.synchronize()
    assert torch.equal(out0[0, k], out1[0, k]) and torch.equal(lse0[0, :, k], lse1[0, :, k])
    assert torch.all(out1[0, 37:] == 0)


def test_unsupported_and_invalid_arguments_are_rejected():
    rng = np.random.default_rng(900)
    wl = _small(rng, 1, 8, 4, 2, 128, [64], "bf16", False)
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    with pytest.raises(api.EtvError):        # P_max beyond the rows the cache holds
        api.tree_verify_attention(d.q, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, m["bitmask"], d.n_nodes,
                                  P_max=10 ** 6)
    # workspace too small for a split launch: five one-tile splits of a 300-key prefix need far more than 256 bytes
    wl5 = _small(rng, 1, 8, 4, 2, 128, [300], "bf16", False)
    d5 = DevWorkload(wl5)
    m5 = api.build_tree_mask(d5.parent, d5.n_nodes)
    need = api.tree_verify_attention_workspace_bytes(api.attn_desc(d5.q, d5.kt, d5.k_cache, None, 300, kv_split=64))
    assert need >= 5 * 8 * 4 * 130 * 4
    with pytest.raises(api.EtvError) as e:
        api.tree_verify_attention(d5.q, d5.k_cache, d5.v_cache, d5.prefix_len, d5.kt, d5.vt, m5["bitmask"], d5.n_nodes,
                                  P_max=300, kv_split=64, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.rc == -3
    q3 = torch.zeros((1, 8, 3, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.EtvError):
        api.tree_verify_attention(q3, d.k_cache, d.v_cache, d.prefix_len, d.kt, d.vt, m["bitmask"], d.n_nodes, P_max=64)


# ---------------------------------------------------------------- the paper-shaped configurations
def test_config2_full_size_contiguous_and_paged():
    for paged in (False, True):
        for qs in (1.0, 4.0):
            wl = synth.config2(paged=paged, with_logits=False, q_scale=qs)
            err, rel = _check(wl)
            print(f"config2 paged={paged} q_scale={qs}: max-abs {err:.3e} scaled {rel:.3e}")


def test_config3_ragged_batch():
    wl = synth.config3(with_logits=False)
    err, rel = _check(wl)
    print(f"config3: max-abs {err:.3e} scaled {rel:.3e}")


def test_config4_long_context_all_heads():
    """Full-size run, every row of every head against the oracle."""
    wl = synth.config4(with_logits=False)
    err, rel = _check(wl, check_lse=True)
    print(f"config4: max-abs {err:.3e} scaled {rel:.3e}")


# the budget sweep: every (T, D) cell; D is clamped to T - 1 (T = 8 with D = 8 or 10 is the depth-7 cell twice)
C5_CELLS = [(T, D) for T in (8, 16, 32, 64, 128) for D in (4, 6, 8, 10)] + [(256, 16)]


@pytest.mark.parametrize("T,D", C5_CELLS)
def test_config5_sweep_cells(T, D):
    """Full batch of 32 on the GPU in the launch shape the benchmark times; the oracle recomputes every row of every
    head of three seeded sequences (the sequences of a cell share one tree and differ in their values)."""
    wl = synth.config5(T, D, with_logits=False)
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    out, _ = gpu_attention(d, m["bitmask"])
    torch.cuda.synchronize()
    ref_mask = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    assert np.array_equal(bits_of(m["bitmask"]).view(np.uint64), ref_mask["bitmask"])
    dense = ref_mask["dense"]
    rng = np.random.default_rng(T * 100 + D)
    for b in sorted(int(x) for x in rng.choice(wl.B, size=3, replace=False)):
        sl = slice(b, b + 1)
        ref, _ = oracle.tree_verify_attention(wl.q[sl], wl.k_cache, wl.v_cache, wl.prefix_len[sl], wl.kt[sl], wl.vt[sl],
                                              dense[sl], wl.n_nodes[sl], dtype="bf16", block_table=wl.block_table[sl])
        err, rel, padded_zero = attention_errors(out[sl], ref, wl.n_nodes[sl])
        _record(f"{wl.name} sequence {b}", err, rel)
        assert padded_zero and err <= TOL["bf16"] and rel <= REL_TOL["bf16"], (T, D, b, err, rel)
