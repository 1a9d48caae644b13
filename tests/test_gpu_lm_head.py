"""GPU parity of lm_head_argmax (teacher head + greedy choice, logits never materialised) against the fp64 oracle.

The argmax is an integer decided by floating point: the kernel accumulates bf16 products in fp32, the oracle in
fp64.  So the index is compared exactly wherever the oracle's two best logits differ by more than the accumulation
error bound, and elsewhere the kernel's choice must be one of the near-maximal entries; exact ties (duplicated weight
rows give bit-identical logits on both sides) must resolve to the lowest index; planted winners must be found."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import api, synth
from gpu_helpers import bits_of, to_dev

pytestmark = pytest.mark.gpu


def _bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _dev_bf16(bits):
    return to_dev(bits).view(torch.bfloat16) if bits.dtype == np.uint16 else to_dev(bits)


def _check(h_bits, w_bits, n, exact=None):
    B, T, D = h_bits.shape
    ref = oracle.lm_head_argmax(h_bits, w_bits, n, dtype="bf16", want_logits=True)
    dh, dw, dn = _dev_bf16(h_bits), _dev_bf16(w_bits), to_dev(np.asarray(n, dtype=np.int32))
    got = api.lm_head_argmax(dh, dw, dn)
    # the same weights packed into tiles: same arithmetic in the same order, so the same bits
    packed = api.pack_lm_head(dw)
    got2 = api.lm_head_argmax(dh, packed, dn, V=w_bits.shape[0])
    torch.cuda.synchronize()
    assert torch.equal(got["argmax"], got2["argmax"]) and torch.equal(got["maxval"], got2["maxval"])
    g, gmax = bits_of(got["argmax"]), bits_of(got["maxval"]).astype(np.float64)
    hf = synth.bf16_bits_to_f32(h_bits).astype(np.float64)
    wf = synth.bf16_bits_to_f32(w_bits).astype(np.float64)
    for b in range(B):
        nb = int(np.clip(n[b], 0, T))
        assert np.all(g[b, nb:] == -1) and np.all(np.isneginf(gmax[b, nb:]))
        for k in range(nb):
            lg = ref["logits"][b, k]
            # fp32 accumulation of D exact products: |error| <= D * 2^-24 * sum |h_c w_vc| for any order
            bound = D * 2.0 ** -24 * float(np.abs(hf[b, k]) @ np.abs(wf[int(g[b, k])])) + 1e-30
            assert 0 <= g[b, k] < w_bits.shape[0]
            assert abs(gmax[b, k] - lg[g[b, k]]) <= bound, (b, k, gmax[b, k], lg[g[b, k]], bound)
            order = np.argsort(-lg, kind="stable")
            margin = lg[order[0]] - lg[order[1]] if len(order) > 1 else np.inf
            if margin > 2 * bound:
                assert g[b, k] == ref["argmax"][b, k], (b, k, margin, bound)
            else:
                assert lg[g[b, k]] >= lg[order[0]] - 2 * bound
    if exact is not None:
        assert np.array_equal(g, exact)
    return ref, g


@pytest.mark.parametrize("B,T,D,V", [(1, 1, 128, 1), (1, 7, 128, 100), (2, 15, 128, 128), (1, 60, 256, 129),
                                      (2, 33, 384, 1000), (3, 60, 128, 700), (1, 128, 128, 513), (2, 128, 256, 300),
                                      (5, 64, 128, 257), (1, 64, 128, 200), (1, 65, 256, 190), (1, 129, 128, 64),
                                      (1, 256, 128, 450)])
def test_random_inputs_all_shapes(B, T, D, V):
    rng = np.random.default_rng(3000 + B * 1000 + T + D + V)
    h = _bf16(rng.standard_normal((B, T, D)))
    w = _bf16(rng.standard_normal((V, D)) / np.sqrt(D))
    n = [T] + [int(rng.integers(0, T + 1)) for _ in range(B - 1)]
    _check(h, w, n)


def test_random_row_counts_and_vocabularies_on_the_wide_path():
    """Seeded sweep over the shapes that exercise the 128-row workgroups: last row groups of 1..127 rows, padded
    sequences, vocabularies that end inside the first or the second half of a tile, one and several tiles."""
    rng = np.random.default_rng(3050)
    for case in range(14):
        B = int(rng.integers(1, 4))
        T = int(rng.integers(max(1, 65 // B), 140))
        D = 128 * int(rng.integers(1, 4))
        V = int(rng.choice([1, 33, 64, 65, 127, 128, 129, 191, 192, 193, 255, 300, 641]))
        h = _bf16(rng.standard_normal((B, T, D)))
        w = _bf16(rng.standard_normal((V, D)) / np.sqrt(D))
        n = [T] + [int(rng.integers(0, T + 1)) for _ in range(B - 1)]
        assert B * T > 64
        _check(h, w, n)


def test_random_row_counts_and_vocabularies_on_the_gemm_path():
    """Beyond 256 node rows the head runs as a GEMM tiling (256 vocabulary rows x 256 node rows per workgroup): row
    counts that end inside the first, second, third or fourth 64-row block of the last row group, padded sequences,
    vocabularies that end inside the first or the second 128-row half of a 256-row tile, one and several tiles,
    contraction lengths of one to three packed steps."""
    rng = np.random.default_rng(3060)
    shapes = [(4, 128, 128, 513), (3, 200, 256, 300), (9, 100, 128, 129), (32, 33, 384, 1000), (2, 256, 128, 256),
              (5, 103, 256, 127), (8, 65, 128, 770), (1, 600, 128, 1), (6, 97, 384, 385), (1, 257, 128, 300),
              (8, 60, 256, 641), (3, 111, 128, 64)]
    for (B, T, D, V) in shapes:
        assert B * T > 256
        h = _bf16(rng.standard_normal((B, T, D)))
        w = _bf16(rng.standard_normal((V, D)) / np.sqrt(D))
        n = [T] + [int(rng.integers(0, T + 1)) for _ in range(B - 1)]
        _check(h, w, n)


def test_exact_ties_on_the_gemm_path_take_the_lowest_index():
    rng = np.random.default_rng(3110)
    B, T, D, V = 5, 128, 128, 900
    hb = _bf16(rng.standard_normal((B, T, D)))
    wb = _bf16(rng.standard_normal((V, D)) / np.sqrt(D))
    hf = synth.bf16_bits_to_f32(hb)
    # node (2, 77): a clear winner duplicated in another 256-row tile, in the other 128-row half of its tile, in
    # another 32-row block of its half and in the last (partial) tile
    win = _bf16(8.0 * hf[2, 77] / float(hf[2, 77] @ hf[2, 77]))
    for v in (300, 37, 310, 420, 899):
        wb[v] = win
    ref, g = _check(hb, wb, [T] * B)
    assert g[2, 77] == 37 and ref["argmax"][2, 77] == 37
    wb[37] = _bf16(rng.standard_normal(D) / np.sqrt(D))
    ref, g = _check(hb, wb, [T] * B)
    assert g[2, 77] == 300


def test_unsupported_width_is_rejected():
    h = torch.zeros((1, 4, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((10, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.EtvError):
        api.lm_head_argmax(h, w, torch.ones(1, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("T", [40, 100])     # 100 rows: the 128-row workgroups that take a tile in two passes
def test_exact_ties_take_the_lowest_index_within_and_across_tiles(T):
    rng = np.random.default_rng(3100)
    B, D, V = 1, 128, 600
    h = rng.standard_normal((B, T, D)).astype(np.float32)
    w = (rng.standard_normal((V, D)) / np.sqrt(D)).astype(np.float32)
    hb = _bf16(h)
    wb = _bf16(w)
    hf = synth.bf16_bits_to_f32(hb)
    # make row 300 a clear winner for node 0 and duplicate it at 37 (another tile), 310 (same tile, same 32-block),
    # 350 (same tile, other block; the other half of the tile) and 599 (last tile): bit-identical logits, the
    # lowest index must win
    win = _bf16(8.0 * hf[0, 0] / float(hf[0, 0] @ hf[0, 0]))
    for v in (300, 37, 310, 350, 599):
        wb[v] = win
    ref, g = _check(hb, wb, [T])
    assert g[0, 0] == 37 and ref["argmax"][0, 0] == 37
    # and with the duplicates only above 300
    wb[37] = _bf16(w[37])
    ref, g = _check(hb, wb, [T])
    assert g[0, 0] == 300


def test_planted_winners_at_verify_step_size():
    rng = np.random.default_rng(3200)
    for (B, T, D, V) in ((1, 60, 1024, 32000), (1, 60, 4096, 2048), (2, 60, 512, 4000), (1, 128, 1024, 8000)):
        h = rng.standard_normal((B, T, D)).astype(np.float32)
        w = (rng.standard_normal((V, D)) / np.sqrt(D)).astype(np.float32)
        hb = _bf16(h)
        hf = synth.bf16_bits_to_f32(hb).astype(np.float64)
        target = rng.permutation(V)[: B * T].reshape(B, T)
        for b in range(B):
            for k in range(T):
                w[target[b, k]] = (12.0 * hf[b, k] / (hf[b, k] @ hf[b, k])).astype(np.float32)
        _check(hb, _bf16(w), [T] * B, exact=target.astype(np.int32))


def test_head_to_commit_without_logits():
    """hidden states -> lm_head_argmax -> the fused epilogue taking the per-node choice in place of logits: the
    acceptance and the commit equal the oracle's, which is given logits whose row argmax is the oracle head's."""
    from gpu_helpers import DevWorkload
    from helpers import logits_from_argmax
    rng = np.random.default_rng(3300)
    wl = synth.config2(P=300, with_logits=False)
    B, T, D, V = wl.B, wl.T_max, 512, wl.V
    h = rng.standard_normal((B, T, D)).astype(np.float32)
    w = (rng.standard_normal((V, D)) / np.sqrt(D)).astype(np.float32)
    hb = _bf16(h)
    hf = synth.bf16_bits_to_f32(hb).astype(np.float64)
    # the teacher agrees with the draft along one root-to-leaf path for three steps, then picks something else
    path = [int(x) for x in wl.retrieve[0, 5] if x >= 0]
    plant = {path[i]: int(wl.tokens[0, path[i + 1]]) for i in range(min(3, len(path) - 1))}
    free = [int(x) for x in rng.permutation(V) if int(x) not in set(plant.values())]
    for node in range(T):
        v = plant.get(node, free[node])      # distinct rows, so every node keeps its planted winner
        w[v] = (12.0 * hf[0, node] / (hf[0, node] @ hf[0, node])).astype(np.float32)
    wb = _bf16(w)
    ref_head = oracle.lm_head_argmax(hb, wb, wl.n_nodes, dtype="bf16")
    lg = np.stack([logits_from_argmax(rng, ref_head["argmax"][b].clip(0), V) for b in range(B)])
    rp = oracle.evaluate_posterior(lg, wl.tokens, wl.retrieve, wl.n_nodes)
    kc, vc = wl.k_cache[None].copy(), wl.v_cache[None].copy()
    rc = oracle.commit_accepted_kv(wl.kt[None], wl.vt[None], kc, vc, wl.prefix_len, wl.capacity, wl.n_nodes,
                                   rp["acc_nodes"], rp["accept_len"], block_table=wl.block_table)
    assert rp["accept_len"][0] >= 1

    d = DevWorkload(wl)
    head = api.lm_head_argmax(_dev_bf16(hb), api.pack_lm_head(_dev_bf16(wb)), d.n_nodes, V=V)
    dkc, dvc = d.k_cache[None].clone(), d.v_cache[None].clone()
    g, p, c = api.verify_epilogue(None, d.tokens, d.retrieve, d.n_nodes, d.kt[None], d.vt[None], dkc, dvc,
                                  d.prefix_len, d.capacity, block_table=d.block_table,
                                  post_out=dict(argmax=head["argmax"]))
    p2 = api.evaluate_posterior(None, d.tokens, d.retrieve, d.n_nodes, out=dict(argmax=head["argmax"]))
    # third way: the head stops after its weight pass and the epilogue finishes the choice per node itself
    part = api.lm_head_argmax(_dev_bf16(hb), _dev_bf16(wb), d.n_nodes, finish=False)
    dkc3, dvc3 = d.k_cache[None].clone(), d.v_cache[None].clone()
    g3, p3, c3 = api.verify_epilogue(None, d.tokens, d.retrieve, d.n_nodes, d.kt[None], d.vt[None], dkc3, dvc3,
                                     d.prefix_len, d.capacity, block_table=d.block_table,
                                     workspace=part["workspace"], head_V=V)
    p4 = api.evaluate_posterior(None, d.tokens, d.retrieve, d.n_nodes, workspace=part["workspace"], head_V=V)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(p3["argmax"])[0, :int(wl.n_nodes[0])], ref_head["argmax"][0, :int(wl.n_nodes[0])])
    assert np.all(bits_of(p3["argmax"])[0, int(wl.n_nodes[0]):] == -1)
    for key in ("len", "best", "accept_len", "acc_nodes", "bonus"):
        assert np.array_equal(bits_of(p3[key]), rp[key]) and np.array_equal(bits_of(p4[key]), rp[key]), key
    for key in rc:
        assert np.array_equal(bits_of(c3[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc3), kc) and np.array_equal(bits_of(dvc3), vc)
    n = int(wl.n_nodes[0])
    assert np.array_equal(bits_of(head["argmax"])[0, :n], ref_head["argmax"][0, :n])
    for key in ("len", "best", "accept_len", "acc_nodes", "bonus"):
        assert np.array_equal(bits_of(p[key]), rp[key]), key
        assert np.array_equal(bits_of(p2[key]), rp[key]), key
    for key in rc:
        assert np.array_equal(bits_of(c[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc), kc) and np.array_equal(bits_of(dvc), vc)
