"""GPU parity (bit-exact) for build_tree_mask, tensorize_tree, safe_gather_paths, evaluate_posterior, commit_accepted_kv."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import api, synth
from gpu_helpers import DEV, DevWorkload, bits_of, to_dev
from helpers import golden, logits_from_argmax, random_tree

pytestmark = pytest.mark.gpu


def _mask_case(parents_np, n_np):
    ref = oracle.build_tree_mask(parents_np, n_np)
    got = api.build_tree_mask(to_dev(parents_np.astype(np.int32)), to_dev(np.asarray(n_np, dtype=np.int32)))
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(got["bitmask"]).view(np.uint64), ref["bitmask"])
    assert np.array_equal(bits_of(got["dense"]), ref["dense"])
    assert np.array_equal(bits_of(got["depth"]), ref["depth"])
    assert np.array_equal(bits_of(got["status"]), ref["status"])
    return ref


@pytest.mark.parametrize("T", [1, 2, 7, 15, 60, 64, 65, 127, 128, 200, 256])
def test_mask_random_trees(T):
    rng = np.random.default_rng(1000 + T)
    B = 9
    par = np.zeros((B, T), dtype=np.int32)
    n = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n[b] = T if b < 3 else rng.integers(0, T + 1)
        par[b, : n[b]] = random_tree(rng, max(1, int(n[b])))[: n[b]]
        par[b, n[b]:] = rng.integers(-5, T + 5, size=T - n[b])   # garbage in padding
    ref = _mask_case(par, n)
    assert np.all(ref["status"] == 0)


def _tensorize_case(parents_np, n_np, P_np, L_max, W):
    ref = oracle.tensorize_tree(parents_np, n_np, P_np, L_max, W)
    refm = oracle.build_tree_mask(parents_np, n_np)
    got = api.tensorize_tree(to_dev(parents_np.astype(np.int32)), to_dev(np.asarray(n_np, dtype=np.int32)),
                             to_dev(np.asarray(P_np, dtype=np.int32)), L_max, W)
    torch.cuda.synchronize()
    for name in ("depth", "position_ids", "retrieve", "n_paths", "status"):
        assert np.array_equal(bits_of(got[name]), ref[name]), name
    assert np.array_equal(bits_of(got["bitmask"]).view(np.uint64), refm["bitmask"])
    assert np.array_equal(bits_of(got["dense"]), refm["dense"])
    return ref


@pytest.mark.parametrize("T", [1, 2, 7, 15, 60, 64, 65, 127, 128, 200, 256])
def test_tensorize_random_trees(T):
    rng = np.random.default_rng(2000 + T)
    B = 9
    par = np.zeros((B, T), dtype=np.int32)
    n = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n[b] = T if b < 3 else rng.integers(0, T + 1)
        par[b, : n[b]] = random_tree(rng, max(1, int(n[b])))[: n[b]]
        par[b, n[b]:] = rng.integers(-5, T + 5, size=T - n[b])   # garbage in padding
    P = rng.integers(-3, 100000, size=B)
    ref = _tensorize_case(par, n, P, T, T)                        # room for every leaf and every depth
    assert np.all(ref["status"] == 0)
    _tensorize_case(par, n, P, max(1, T // 3), max(1, T // 4))   # overflow of both kinds on most sequences
    _tensorize_case(par, n, P, 1, 1)


def test_tensorize_shapes_of_the_workloads_invalid_trees_and_worked_example():
    ex = golden("worked_example.json")
    ref = _tensorize_case(np.asarray([ex["parent"]], dtype=np.int32), [7], [100], 4, 4)
    assert ref["retrieve"][0, :3].tolist() == ex["retrieve"]
    # chain, star, and the generators of the paper-shaped workloads: the device table equals the host-built one
    for par, W in ((synth.tree_chain(128), 128), (synth.tree_star(128), 2),
                   (synth.tree_eagle(np.random.default_rng(3), 60, 6, 10), 7),
                   (synth.tree_bfs(np.random.default_rng(4), 128, 8, 4), 9),
                   (synth.tree_spine_leaves(64, 8, 4), 9)):
        T = len(par)
        host = synth.build_retrieve(par, W)
        ref = _tensorize_case(par[None].astype(np.int32), [T], [4096], host.shape[0] + 2, W)
        assert ref["n_paths"][0] == host.shape[0] and ref["status"][0] == 0
        assert np.array_equal(ref["retrieve"][0, :host.shape[0]], host)
    rng = np.random.default_rng(6)
    T, B = 40, 64
    par = np.stack([random_tree(rng, T) for _ in range(B)])
    n = np.full(B, T, dtype=np.int32)
    for b in range(B):
        kind = b % 4
        k = int(rng.integers(1, T))
        if kind == 0:
            par[b, k] = rng.choice([-1, -7, T, T + 3, 2 ** 30])
        elif kind == 1:
            j = int(rng.integers(1, T))
            par[b, k] = j; par[b, j] = k            # 2-cycle (or self loop when j == k)
        elif kind == 2:
            n[b] = T - 5; par[b, int(rng.integers(1, T - 5))] = T - 2   # parent in the padded region
        else:
            par[b, 0] = 3
    ref = _tensorize_case(par, n, np.zeros(B), T, T)
    assert np.all(ref["status"] != 0)


def test_mask_invalid_trees_and_worked_example():
    ex = golden("worked_example.json")
    ref = _mask_case(np.asarray([ex["parent"]], dtype=np.int32), [7])
    assert ref["bitmask"][0, :, 0].tolist() == ex["bitmask_words"]
    rng = np.random.default_rng(5)
    T, B = 40, 64
    par = np.stack([random_tree(rng, T) for _ in range(B)])
    n = np.full(B, T, dtype=np.int32)
    for b in range(B):
        kind = b % 4
        k = int(rng.integers(1, T))
        if kind == 0:
            par[b, k] = rng.choice([-1, -7, T, T + 3, 2 ** 30])
        elif kind == 1:
            j = int(rng.integers(1, T))
            par[b, k] = j; par[b, j] = k            # 2-cycle (or self loop when j == k)
        elif kind == 2:
            n[b] = T - 5; par[b, int(rng.integers(1, T - 5))] = T - 2   # parent in the padded region
        else:
            par[b, 0] = 3
    ref = _mask_case(par, n)
    assert np.all(ref["status"] != 0)


def test_mask_workload_trees():
    for wl in (synth.config1(), synth.config2(with_cache=False, with_logits=False),
               synth.config3(with_cache=False, with_logits=False), synth.config4(with_cache=False, with_logits=False),
               synth.config5(128, 10, with_cache=False, with_logits=False),
               synth.config5(8, 10, with_cache=False, with_logits=False)):
        _mask_case(wl.parent, wl.n_nodes)


def test_safe_gather_matches_oracle_and_rejects_bad_dummy():
    rng = np.random.default_rng(21)
    for (B, L, W, T_max, shape, dt) in [(3, 6, 5, 9, (3,), np.float32), (2, 40, 7, 60, (), np.int32),
                                        (4, 11, 11, 128, (5, 2), np.uint8), (2, 5, 4, 16, (64,), np.float32),
                                        (1, 3, 4, 7, (4096,), np.uint16)]:
        ret = rng.integers(-3, T_max + 3, size=(B, L, W)).astype(np.int32)
        n = rng.integers(0, T_max + 1, size=B).astype(np.int32)
        Z = rng.integers(0, 255, size=(B, T_max) + shape).astype(dt)
        for dummy in (0, T_max - 1):
            ref = oracle.safe_gather_paths(ret, n, T_max, dummy, Z)
            got = api.safe_gather_paths(to_dev(ret), to_dev(n), T_max, dummy, to_dev(Z) if dt != np.uint16
                                        else torch.from_numpy(Z.view(np.int16)).to(DEV))
            torch.cuda.synchronize()
            assert np.array_equal(bits_of(got["safe"]), ref["safe"])
            assert np.array_equal(bits_of(got["pvalid"]), ref["pvalid"])
            assert np.array_equal(bits_of(got["gathered"]).view(dt), ref["gathered"])
            assert got["safe"].min().item() >= 0
    ret_d, n_d = to_dev(ret), to_dev(n)
    for bad in (-1, T_max):
        with pytest.raises(api.EtvError):
            api.safe_gather_paths(ret_d, n_d, T_max, bad)


def _posterior_case(logits, tokens, retrieve, n, dummy=0):
    ref = oracle.evaluate_posterior(logits, tokens, retrieve, n, dummy)
    got = api.evaluate_posterior(to_dev(logits), to_dev(tokens), to_dev(retrieve), to_dev(np.asarray(n, np.int32)), dummy)
    torch.cuda.synchronize()
    for key in ("argmax", "len", "best", "accept_len", "acc_nodes", "bonus"):
        assert np.array_equal(bits_of(got[key]), ref[key]), key
    return ref


def test_posterior_worked_example_and_trap():
    ex = golden("worked_example.json")
    rng = np.random.default_rng(22)
    ret = np.asarray([ex["retrieve"]], dtype=np.int32)
    tok = np.asarray([ex["tokens"]], dtype=np.int32)
    for case in ("case_main", "case_trap"):
        lg = logits_from_argmax(rng, ex[case]["argmax"], 128)[None]
        ref = _posterior_case(lg, tok, ret, [7])
        assert int(ref["accept_len"][0]) == ex[case]["accept_len"] and ref["acc_nodes"][0].tolist() == ex[case]["acc_nodes"]


@pytest.mark.parametrize("V", [5, 16, 1000, 4096, 4097, 32000, 50257])
def test_posterior_random_small_vocab_many_matches(V):
    rng = np.random.default_rng(300 + V)
    B, T = 5, 24
    parents = [random_tree(rng, int(rng.integers(1, T + 1))) for _ in range(B)]
    Vt = max(V, 24)
    wl = synth.assemble("t", rng, parents, [8] * B, Hq=1, Hkv=1, d=8, dtype="f32", V=Vt, W=T, paged=False, T_max=T,
                        with_cache=False, with_logits=False)
    lg = rng.standard_normal((B, T, Vt)).astype(np.float32)
    if V <= 16:                                         # quantise => ties inside rows, tokens within a tiny range
        lg = np.round(lg)
        wl.tokens %= V
    lg[:, :, Vt - 1] += (rng.random((B, T)) < 0.2) * 30  # maxima at the very end of the row
    lg[0, 0, :] = -np.inf                                # an all -inf row: argmax = 0
    for dummy in (0, 3):
        _posterior_case(lg, wl.tokens, wl.retrieve, wl.n_nodes, dummy)


def test_posterior_workloads_with_planted_paths():
    for wl in (synth.config1(), synth.config2(with_cache=False), synth.config3(with_cache=False),
               synth.config5(64, 10, B=6, with_cache=False)):
        ref = _posterior_case(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes)
        assert ref["accept_len"].tolist() == [a for _, a in wl.planted]


def _commit_case(wl, Lyr, A, acc, capacity=None):
    rng = np.random.default_rng(77)
    dt = wl.dtype
    kt = np.stack([synth._values(rng, wl.kt.shape, dt) for _ in range(Lyr)])
    vt = np.stack([synth._values(rng, wl.vt.shape, dt) for _ in range(Lyr)])
    kc = np.stack([synth._values(rng, wl.k_cache.shape, dt) for _ in range(Lyr)])
    vc = np.stack([synth._values(rng, wl.v_cache.shape, dt) for _ in range(Lyr)])
    cap = wl.capacity if capacity is None else capacity
    d_kc, d_vc = to_dev(kc), to_dev(vc)
    got = api.commit_accepted_kv(to_dev(kt), to_dev(vt), d_kc, d_vc, to_dev(wl.prefix_len), to_dev(cap),
                                 to_dev(wl.n_nodes), to_dev(acc), to_dev(np.asarray(A, np.int32)),
                                 block_table=to_dev(wl.block_table))
    torch.cuda.synchronize()
    ref = oracle.commit_accepted_kv(kt, vt, kc, vc, wl.prefix_len, cap, wl.n_nodes, acc, A, block_table=wl.block_table)
    for key in ("prefix_len_out", "slot_map", "status"):
        assert np.array_equal(bits_of(got[key]), ref[key]), key
    assert np.array_equal(bits_of(d_kc), kc) and np.array_equal(bits_of(d_vc), vc)   # whole cache, every byte
    return ref


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_commit_matches_oracle_including_failures(paged, dtype):
    rng = np.random.default_rng(41)
    B, T, W = 6, 12, 12
    parents = [random_tree(rng, T) for _ in range(B)]
    wl = synth.assemble("t", rng, parents, [20, 16, 15, 33, 0, 47], Hq=4, Hkv=4, d=64, dtype=dtype, V=512, W=W,
                        paged=paged, with_logits=False, spare_blocks=4)
    acc = np.zeros((B, W), dtype=np.int32)
    A = np.zeros(B, dtype=np.int32)
    for b in range(B):
        path = wl.retrieve[b, b % wl.n_paths[b]]
        A[b] = min(b, int((path >= 0).sum()) - 1)
        acc[b, : A[b] + 1] = path[: A[b] + 1]
    ref = _commit_case(wl, 3, A, acc)
    assert np.all(ref["status"] == 0)
    cap = wl.capacity.copy(); cap[1] = wl.prefix_len[1] + A[1]      # one row short
    acc2 = acc.copy(); acc2[2, 0] = T + 1                            # invalid node
    A2 = A.copy(); A2[3] = W; A2[5] = -2
    ref = _commit_case(wl, 2, A2, acc2, cap)
    assert ref["status"].tolist() == [0, api.COMMIT_CAPACITY, api.COMMIT_BAD_NODE, api.COMMIT_BAD_LEN, 0,
                                      api.COMMIT_BAD_LEN]


def test_commit_fully_accepted_chain_and_aliasing_prefix_len():
    rng = np.random.default_rng(42)
    T, P = 9, 30
    wl = synth.assemble("t", rng, [synth.tree_chain(T)], [P], Hq=8, Hkv=8, d=128, dtype="bf16", V=512, W=T, paged=True,
                        with_logits=False)
    acc = np.arange(T, dtype=np.int32)[None]
    ref = _commit_case(wl, 4, [T - 1], acc)
    assert int(ref["prefix_len_out"][0]) == P + T
    # prefix_len_out may alias prefix_len
    kt, vt = to_dev(wl.kt[None]), to_dev(wl.vt[None])
    kc, vc = to_dev(wl.k_cache[None]), to_dev(wl.v_cache[None])
    plen = to_dev(wl.prefix_len)
    got = api.commit_accepted_kv(kt, vt, kc, vc, plen, to_dev(wl.capacity), to_dev(wl.n_nodes), to_dev(acc),
                                 to_dev(np.asarray([T - 1], np.int32)), block_table=to_dev(wl.block_table),
                                 prefix_len_out=plen)
    torch.cuda.synchronize()
    assert plen.item() == P + T and np.array_equal(bits_of(got["slot_map"]), ref["slot_map"])


def test_probe_library_runs_and_rejects_bad_arguments():
    """The measurement aids (their own library): the stream probe only reads, the MFMA probe touches no memory."""
    from paper_2603_08088_amd import probe
    buf = torch.ones(8 * 2 ** 20, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda:0")
    probe.hbm_read_probe(buf, sink)
    probe.mfma_bf16_probe(4, sink)
    probe.mfma_bf16_live_probe(3, sink)
    torch.cuda.synchronize()
    assert int(sink.sum().item()) == 0
    assert probe.mfma_bf16_live_probe_flops(66) == 512 * 8 * 66 * 32 * 2.0 * 32 * 32 * 16
    with pytest.raises(RuntimeError):
        probe.hbm_read_probe(buf[: 2 ** 16], sink)   # below the 1 MiB minimum
    with pytest.raises(RuntimeError):
        probe.hbm_read_probe(buf[1:], sink)          # misaligned
    with pytest.raises(RuntimeError):
        probe.mfma_bf16_probe(0, sink)
    with pytest.raises(RuntimeError):
        probe.mfma_bf16_live_probe(0, sink)


def _epilogue_case(wl, L=2, dummy=0, spoil=None):
    """The fused epilogue against the oracle's gather, acceptance and commit (and so against the separate calls)."""
    rng = np.random.default_rng(77)
    kt = np.stack([wl.kt] + [synth._values(rng, wl.kt.shape, wl.dtype) for _ in range(L - 1)])
    vt = np.stack([wl.vt] + [synth._values(rng, wl.vt.shape, wl.dtype) for _ in range(L - 1)])
    kc = np.stack([wl.k_cache] + [synth._values(rng, wl.k_cache.shape, wl.dtype) for _ in range(L - 1)])
    vc = np.stack([wl.v_cache] + [synth._values(rng, wl.v_cache.shape, wl.dtype) for _ in range(L - 1)])
    capacity = wl.capacity.copy()
    if spoil is not None:
        capacity[spoil] = wl.prefix_len[spoil]          # no room: that sequence must be left untouched
    tok3 = wl.tokens.reshape(wl.B, wl.T_max, 1)
    rg = oracle.safe_gather_paths(wl.retrieve, wl.n_nodes, wl.T_max, dummy, tok3)
    rp = oracle.evaluate_posterior(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes, dummy)
    okc, ovc = kc.copy(), vc.copy()
    rc = oracle.commit_accepted_kv(kt, vt, okc, ovc, wl.prefix_len, capacity, wl.n_nodes, rp["acc_nodes"],
                                   rp["accept_len"], block_table=wl.block_table)
    d = DevWorkload(wl)
    dkc, dvc = to_dev(kc), to_dev(vc)
    g, p, c = api.verify_epilogue(d.logits, d.tokens, d.retrieve, d.n_nodes, to_dev(kt), to_dev(vt), dkc, dvc,
                                  d.prefix_len, to_dev(capacity), block_table=d.block_table, dummy=dummy,
                                  src=d.tokens.reshape(wl.B, wl.T_max, 1))
    torch.cuda.synchronize()
    for key in ("safe", "pvalid", "gathered"):
        assert np.array_equal(bits_of(g[key]), rg[key]), key
    for key in rp:
        assert np.array_equal(bits_of(p[key]), rp[key]), key
    for key in rc:
        assert np.array_equal(bits_of(c[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    return rp, rc


def test_fused_epilogue_matches_gather_acceptance_and_commit():
    rp, rc = _epilogue_case(synth.config1())
    assert np.all(rc["status"] == 0)
    for paged in (False, True):
        rp, rc = _epilogue_case(synth.config2(paged=paged, P=300))
        assert np.all(rc["status"] == 0)
    rp, rc = _epilogue_case(synth.config3(B=4, lo=100, hi=600), spoil=2)     # ragged, paged, one sequence out of room
    assert rc["status"][2] != 0 and np.all(np.delete(rc["status"], 2) == 0)
    assert len(set(rp["accept_len"].tolist())) > 1
    _epilogue_case(synth.config5(16, 4, B=6, P=200), dummy=3)               # padding-heavy path table, dummy != 0


@pytest.mark.parametrize("paged", [False, True])
def test_in_place_branch_cache_attention_and_commit(paged):
    """The tree K/V live in the cache itself behind the prefix (no separate tree buffer): attention must give the
    bits it gives with the separate buffer, and the commit must compact the accepted rows as the oracle does,
    through the plain and the fused entry points, including destinations that were sources of earlier rows."""
    from gpu_helpers import gpu_attention
    rng = np.random.default_rng(88)
    B, T, L = 5, 40, 2
    parents = [random_tree(rng, T) for _ in range(B)]
    wl = synth.assemble("tail", rng, parents, [300, 77, 64, 1, 129], Hq=8, Hkv=2, d=128, dtype="bf16", V=512, W=T,
                        paged=paged, T_max=T, spare_blocks=3, tail_room=T)
    wl.n_nodes[1] = 17                                   # one padded sequence
    kt = np.stack([wl.kt] + [synth._values(rng, wl.kt.shape, "bf16") for _ in range(L - 1)])
    vt = np.stack([wl.vt] + [synth._values(rng, wl.vt.shape, "bf16") for _ in range(L - 1)])
    kc = np.stack([wl.k_cache] + [synth._values(rng, wl.k_cache.shape, "bf16") for _ in range(L - 1)])
    vc = np.stack([wl.v_cache] + [synth._values(rng, wl.v_cache.shape, "bf16") for _ in range(L - 1)])
    for b in range(B):                                   # the verification pass has extended the cache in place
        for j in range(int(wl.n_nodes[b])):
            pos = int(wl.prefix_len[b]) + j
            if paged:
                blk, off = wl.block_table[b, pos // synth.BLOCK], pos % synth.BLOCK
                kc[:, blk, :, off] = kt[:, b, j]; vc[:, blk, :, off] = vt[:, b, j]
            else:
                kc[:, b, pos] = kt[:, b, j]; vc[:, b, pos] = vt[:, b, j]
    wl.k_cache, wl.v_cache = kc[0].copy(), vc[0].copy()
    d = DevWorkload(wl)
    m = api.build_tree_mask(d.parent, d.n_nodes)
    for kw in (dict(), dict(kv_split=64), dict(flags=api.ATTN_FLAG_GENERIC)):
        sep, lse_sep = gpu_attention(d, m["bitmask"], **kw)
        tail, lse_tail = api.tree_verify_attention(d.q, d.k_cache, d.v_cache, d.prefix_len, None, None, m["bitmask"],
                                                   d.n_nodes, P_max=d.P_max, block_table=d.block_table, **kw)
        torch.cuda.synchronize()
        assert torch.equal(sep, tail) and torch.equal(lse_sep, lse_tail), kw
    # commit: full accepted paths of different leaves
    acc = np.zeros((B, T), dtype=np.int32)
    A = np.zeros(B, dtype=np.int32)
    for b in range(B):
        path = [int(x) for x in wl.retrieve[b, b % wl.n_paths[b]] if 0 <= x < wl.n_nodes[b]]
        A[b] = len(path) - 1
        acc[b, :len(path)] = path
    okc, ovc = kc.copy(), vc.copy()
    rc = oracle.commit_accepted_kv(None, None, okc, ovc, wl.prefix_len, wl.capacity, wl.n_nodes, acc, A,
                                   block_table=wl.block_table, T_max=T)
    assert np.all(rc["status"] == 0)
    dkc, dvc = to_dev(kc), to_dev(vc)
    c = api.commit_accepted_kv(None, None, dkc, dvc, d.prefix_len, d.capacity, d.n_nodes, to_dev(acc), to_dev(A),
                               block_table=d.block_table, T_max=T)
    torch.cuda.synchronize()
    for key in rc:
        assert np.array_equal(bits_of(c[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    # a sequence without room for its tail is refused and left alone
    cap = wl.capacity.copy(); cap[0] = wl.prefix_len[0] + 3
    okc2, ovc2 = kc.copy(), vc.copy()
    rc2 = oracle.commit_accepted_kv(None, None, okc2, ovc2, wl.prefix_len, cap, wl.n_nodes, acc, A,
                                    block_table=wl.block_table, T_max=T)
    dkc2, dvc2 = to_dev(kc), to_dev(vc)
    c2 = api.commit_accepted_kv(None, None, dkc2, dvc2, d.prefix_len, to_dev(cap), d.n_nodes, to_dev(acc), to_dev(A),
                                block_table=d.block_table, T_max=T)
    torch.cuda.synchronize()
    assert rc2["status"][0] != 0
    for key in rc2:
        assert np.array_equal(bits_of(c2[key]), rc2[key]), key
    assert np.array_equal(bits_of(dkc2), okc2) and np.array_equal(bits_of(dvc2), ovc2)
    # the fused epilogue over the in-place branch cache: acceptance from the logits, then compaction
    rp = oracle.evaluate_posterior(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes)
    okc3, ovc3 = kc.copy(), vc.copy()
    rc3 = oracle.commit_accepted_kv(None, None, okc3, ovc3, wl.prefix_len, wl.capacity, wl.n_nodes, rp["acc_nodes"],
                                    rp["accept_len"], block_table=wl.block_table, T_max=T)
    dkc3, dvc3 = to_dev(kc), to_dev(vc)
    g3, p3, c3 = api.verify_epilogue(d.logits, d.tokens, d.retrieve, d.n_nodes, None, None, dkc3, dvc3, d.prefix_len,
                                     d.capacity, block_table=d.block_table)
    torch.cuda.synchronize()
    for key in rp:
        assert np.array_equal(bits_of(p3[key]), rp[key]), key
    for key in rc3:
        assert np.array_equal(bits_of(c3[key]), rc3[key]), key
    assert np.array_equal(bits_of(dkc3), okc3) and np.array_equal(bits_of(dvc3), ovc3)


@pytest.mark.parametrize("paged", [False, True])
def test_in_place_commit_of_a_deep_gapped_path_and_refusal_of_a_backward_path(paged):
    """An accepted path of 24 rows (more than one batch of sixteen) with gaps, so that sources of the second batch lie
    just above destinations of the first, over five layers: the plain call and the fused epilogue (teacher choices
    given per node) must leave the cache as the oracle's gather from a snapshot does.  A path that does not walk
    the tail front to back is refused by both sides and the sequence stays untouched."""
    rng = np.random.default_rng(91)
    T, L = 40, 5
    path = [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 17, 18, 20, 23, 27, 31, 36, 39]
    par = np.zeros(T, dtype=np.int32)
    for a, c in zip(path[:-1], path[1:]):
        par[c] = a
    par2 = par.copy(); par2[16] = 3                        # second sequence: same spine, node 16 deeper in
    wl = synth.assemble("deep_tail", rng, [par, par2, par], [21, 64, 5], Hq=4, Hkv=2, d=128, dtype="bf16", V=512, W=T,
                        paged=paged, T_max=T, spare_blocks=3, tail_room=T, with_logits=False)
    kc = np.stack([synth._values(rng, wl.k_cache.shape, "bf16") for _ in range(L)])
    vc = np.stack([synth._values(rng, wl.v_cache.shape, "bf16") for _ in range(L)])
    d = DevWorkload(wl)
    acc = np.zeros((3, T), dtype=np.int32)
    acc[0, :24] = path; acc[1, :24] = path
    acc[2, :4] = [0, 2, 1, 3]                              # goes back: refused in place
    A = np.array([23, 23, 3], dtype=np.int32)
    okc, ovc = kc.copy(), vc.copy()
    rc = oracle.commit_accepted_kv(None, None, okc, ovc, wl.prefix_len, wl.capacity, wl.n_nodes, acc, A,
                                   block_table=wl.block_table, T_max=T)
    assert rc["status"].tolist() == [0, 0, api.COMMIT_BAD_NODE]
    assert not np.array_equal(okc, kc)
    dkc, dvc = to_dev(kc), to_dev(vc)
    c = api.commit_accepted_kv(None, None, dkc, dvc, d.prefix_len, d.capacity, d.n_nodes, to_dev(acc), to_dev(A),
                               block_table=d.block_table, T_max=T)
    torch.cuda.synchronize()
    for key in rc:
        assert np.array_equal(bits_of(c[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    # fused epilogue: the teacher's choice per node is given, planted so that the whole spine is accepted
    g = np.full((3, T), -1, dtype=np.int32)
    for b in range(3):
        for a_, c_ in zip(path[:-1], path[1:]):
            g[b, a_] = wl.tokens[b, c_]
        g[b, path[-1]] = 7
    g[g < 0] = 0                                           # every node has a choice; off the spine it is token 0
    rp = oracle.evaluate_posterior(synth_logits_from(g, 512), wl.tokens, wl.retrieve, wl.n_nodes)
    assert rp["accept_len"].tolist() == [23, 23, 23] and rp["acc_nodes"][0, :24].tolist() == path
    okc2, ovc2 = kc.copy(), vc.copy()
    rc2 = oracle.commit_accepted_kv(None, None, okc2, ovc2, wl.prefix_len, wl.capacity, wl.n_nodes, rp["acc_nodes"],
                                    rp["accept_len"], block_table=wl.block_table, T_max=T)
    assert rc2["status"].tolist() == [0, 0, 0]
    dkc2, dvc2 = to_dev(kc), to_dev(vc)
    _, p2, c2 = api.verify_epilogue(None, d.tokens, d.retrieve, d.n_nodes, None, None, dkc2, dvc2, d.prefix_len,
                                    d.capacity, block_table=d.block_table, post_out=dict(argmax=to_dev(g)))
    torch.cuda.synchronize()
    for key in rp:
        assert np.array_equal(bits_of(p2[key]), rp[key]), key
    for key in rc2:
        assert np.array_equal(bits_of(c2[key]), rc2[key]), key
    assert np.array_equal(bits_of(dkc2), okc2) and np.array_equal(bits_of(dvc2), ovc2)


def synth_logits_from(g, V):
    """Logits whose row argmax is g (padding rows, g < 0: any)."""
    lg = np.zeros(g.shape + (V,), dtype=np.float32)
    for idx in np.ndindex(g.shape):
        if g[idx] >= 0:
            lg[idx][g[idx]] = 5.0
    return lg


def test_fused_epilogue_refuses_an_aliased_prefix_length_output():
    wl = synth.config1()
    d = DevWorkload(wl)
    kc, vc = d.k_cache[None].clone(), d.v_cache[None].clone()
    with pytest.raises(api.EtvError):
        api.verify_epilogue(d.logits, d.tokens, d.retrieve, d.n_nodes, d.kt[None], d.vt[None], kc, vc, d.prefix_len,
                            d.capacity, commit_out=dict(prefix_len_out=d.prefix_len))


@pytest.mark.parametrize("in_place", [False, True])
def test_fused_epilogue_on_a_fully_accepted_256_node_chain_and_on_a_batch_of_600(in_place):
    """The extremes of the one-launch epilogue: an accepted path of 256 rows (every thread of the plan has a
    position, the row copy runs over sixteen batches) over three layers, and 600 sequences (one layer group per
    sequence, more acceptance workgroups than compute units)."""
    rng = np.random.default_rng(93 + in_place)
    T, L = 256, 3
    wl = synth.assemble("chain256", rng, [synth.tree_chain(T)], [77], Hq=2, Hkv=2, d=64, dtype="bf16", V=300, W=T,
                        paged=True, T_max=T, spare_blocks=3, tail_room=T, with_logits=False)
    g = np.zeros((1, T), dtype=np.int32)
    g[0, :T - 1] = wl.tokens[0, 1:]                       # every node's choice is its child's token
    g[0, T - 1] = 11
    kc = np.stack([synth._values(rng, wl.k_cache.shape, "bf16") for _ in range(L)])
    vc = np.stack([synth._values(rng, wl.v_cache.shape, "bf16") for _ in range(L)])
    kt = np.stack([synth._values(rng, wl.kt.shape, "bf16") for _ in range(L)])
    vt = np.stack([synth._values(rng, wl.vt.shape, "bf16") for _ in range(L)])
    d = DevWorkload(wl)
    rp = oracle.evaluate_posterior(synth_logits_from(g, 300), wl.tokens, wl.retrieve, wl.n_nodes)
    assert rp["accept_len"].tolist() == [T - 1] and rp["bonus"].tolist() == [11]
    okc, ovc = kc.copy(), vc.copy()
    rc = oracle.commit_accepted_kv(None if in_place else kt, None if in_place else vt, okc, ovc, wl.prefix_len,
                                   wl.capacity, wl.n_nodes, rp["acc_nodes"], rp["accept_len"],
                                   block_table=wl.block_table, T_max=T)
    assert rc["status"].tolist() == [0] and int(rc["prefix_len_out"][0]) == 77 + T
    dkc, dvc = to_dev(kc), to_dev(vc)
    _, p, c = api.verify_epilogue(None, d.tokens, d.retrieve, d.n_nodes, None if in_place else to_dev(kt),
                                  None if in_place else to_dev(vt), dkc, dvc, d.prefix_len, d.capacity,
                                  block_table=d.block_table, post_out=dict(argmax=to_dev(g)))
    torch.cuda.synchronize()
    for key in rp:
        assert np.array_equal(bits_of(p[key]), rp[key]), key
    for key in rc:
        assert np.array_equal(bits_of(c[key]), rc[key]), key
    assert np.array_equal(bits_of(dkc), okc) and np.array_equal(bits_of(dvc), ovc)
    if in_place:
        return
    # 600 short sequences with ragged accept lengths, two layers
    B = 600
    parents = [random_tree(rng, 9) for _ in range(B)]
    wl = synth.assemble("many", rng, parents, [int(x) for x in rng.integers(0, 40, size=B)], Hq=2, Hkv=2, d=64,
                        dtype="bf16", V=64, W=9, paged=True, T_max=9, spare_blocks=3)
    _epilogue_case(wl, L=2)
