"""GPU parity of the whole verify step in the launch configuration bench.py times: full-size config 2,
every entry point through the C ABI, eagerly and as a replayed HIP graph, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_08088_amd import api, synth
from gpu_helpers import DevWorkload, bits_of, to_dev, to_host_f64, attention_errors

pytestmark = pytest.mark.gpu


def _oracle_step(wl, kt, vt, kc, vc, q):
    m = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    m.update({k: v for k, v in oracle.tensorize_tree(wl.parent, wl.n_nodes, wl.prefix_len, wl.retrieve.shape[1],
                                                     wl.W).items() if k not in m})
    assert np.array_equal(m["retrieve"], wl.retrieve)   # the oracle's path table is the generator's
    outs = [oracle.tree_verify_attention(q[l], kc[l], vc[l], wl.prefix_len, kt[l], vt[l], m["dense"], wl.n_nodes,
                                         dtype=wl.dtype, block_table=wl.block_table, want_lse=False)[0]
            for l in range(q.shape[0])]
    g = oracle.safe_gather_paths(wl.retrieve, wl.n_nodes, wl.T_max, 0, wl.tokens.reshape(wl.B, wl.T_max, 1))
    p = oracle.evaluate_posterior(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes)
    kc2, vc2 = kc.copy(), vc.copy()
    c = oracle.commit_accepted_kv(kt, vt, kc2, vc2, wl.prefix_len, wl.capacity, wl.n_nodes, p["acc_nodes"],
                                  p["accept_len"], block_table=wl.block_table)
    return m, outs, g, p, c, kc2, vc2


@pytest.mark.parametrize("paged,fused", [(False, False), (True, False), (False, True), (True, True)])
def test_full_step_config2_eager_and_graph(paged, fused):
    L = 3
    wl = synth.config2(paged=paged)
    rng = np.random.default_rng(99)
    q = np.stack([wl.q] + [synth._values(rng, wl.q.shape, "bf16") for _ in range(L - 1)])
    kt = np.stack([wl.kt] + [synth._values(rng, wl.kt.shape, "bf16") for _ in range(L - 1)])
    vt = np.stack([wl.vt] + [synth._values(rng, wl.vt.shape, "bf16") for _ in range(L - 1)])
    kc = np.stack([wl.k_cache] + [synth._values(rng, wl.k_cache.shape, "bf16") for _ in range(L - 1)])
    vc = np.stack([wl.v_cache] + [synth._values(rng, wl.v_cache.shape, "bf16") for _ in range(L - 1)])
    rm, routs, rg, rp, rc, rkc, rvc = _oracle_step(wl, kt, vt, kc, vc, q)

    d = DevWorkload(wl)
    dq, dkt, dvt = to_dev(q), to_dev(kt), to_dev(vt)
    B, T = wl.B, wl.T_max
    i32 = dict(dtype=torch.int32, device="cuda")
    mask_out = dict(bitmask=torch.empty((B, T, 1), dtype=torch.int64, device="cuda"),
                    dense=torch.empty((B, 1, T, T), dtype=torch.uint8, device="cuda"),
                    depth=torch.empty((B, T), **i32), status=torch.empty((B,), **i32),
                    position_ids=torch.empty((B, T), **i32), n_paths=torch.empty((B,), **i32),
                    retrieve=torch.empty((B,) + wl.retrieve.shape[1:], **i32))
    out = torch.empty_like(dq)
    desc = api.attn_desc(dq[0], dkt[0], to_dev(kc[0]), d.block_table, d.P_max)
    ws = torch.empty(max(256, api.tree_verify_attention_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    L_max, W = wl.retrieve.shape[1], wl.W
    gout = dict(safe=torch.empty((B, L_max, W), **i32), pvalid=torch.empty((B, L_max, W), dtype=torch.uint8, device="cuda"),
                gathered=torch.empty((B, L_max, W, 1), **i32))
    pout = dict(argmax=torch.empty((B, T), **i32), len=torch.empty((B, L_max), **i32), best=torch.empty((B,), **i32),
                accept_len=torch.empty((B,), **i32), acc_nodes=torch.empty((B, W), **i32), bonus=torch.empty((B,), **i32))
    pws = torch.empty(max(256, api.evaluate_posterior_workspace_bytes(B, T, wl.V)), dtype=torch.uint8, device="cuda")
    cout = dict(prefix_len_out=torch.empty((B,), **i32), slot_map=torch.empty((B, W), **i32), status=torch.empty((B,), **i32))

    def step(dkc, dvc):
        # the tree tensors come from the device: the path table the later calls read is the one written here
        api.tensorize_tree(d.parent, d.n_nodes, d.prefix_len, L_max, W, out=mask_out)
        for l in range(L):
            api.tree_verify_attention(dq[l], dkc[l], dvc[l], d.prefix_len, dkt[l], dvt[l], mask_out["bitmask"], d.n_nodes,
                                      P_max=d.P_max, block_table=d.block_table, out=out[l], want_lse=False,
                                      workspace=ws, desc=desc)
        if fused:   # gather + acceptance + commit through the fused epilogue entry point
            api.verify_epilogue(d.logits, d.tokens, mask_out["retrieve"], d.n_nodes, dkt, dvt, dkc, dvc, d.prefix_len,
                                d.capacity, block_table=d.block_table, dummy=0, src=d.tokens.reshape(B, T, 1),
                                workspace=pws, gather_out=gout, post_out=pout, commit_out=cout)
            return
        api.safe_gather_paths(mask_out["retrieve"], d.n_nodes, T, 0, d.tokens.reshape(B, T, 1), out=gout)
        api.evaluate_posterior(d.logits, d.tokens, mask_out["retrieve"], d.n_nodes, 0, workspace=pws, out=pout)
        api.commit_accepted_kv(dkt, dvt, dkc, dvc, d.prefix_len, d.capacity, d.n_nodes, pout["acc_nodes"],
                               pout["accept_len"], block_table=d.block_table, out=cout)

    def check(dkc, dvc, tag):
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(mask_out["dense"]), rm["dense"]), tag
        for key in ("depth", "position_ids", "retrieve", "n_paths", "status"):
            assert np.array_equal(bits_of(mask_out[key]), rm[key]), (tag, key)
        for l in range(L):
            err, rel, pz = attention_errors(out[l], routs[l], wl.n_nodes)
            assert pz and err <= 2e-2 and rel <= 2e-2, (tag, l, err, rel)
        assert np.array_equal(bits_of(gout["safe"]), rg["safe"]) and np.array_equal(bits_of(gout["gathered"]), rg["gathered"])
        for key in rp:
            assert np.array_equal(bits_of(pout[key]), rp[key]), (tag, key)
        for key in rc:
            assert np.array_equal(bits_of(cout[key]), rc[key]), (tag, key)
        assert np.array_equal(bits_of(dkc), rkc) and np.array_equal(bits_of(dvc), rvc), tag

    dkc, dvc = to_dev(kc), to_dev(vc)
    step(dkc, dvc)
    check(dkc, dvc, "eager")

    # the same launches captured once and replayed: every replay must reproduce the eager results
    dkc2, dvc2 = to_dev(kc), to_dev(vc)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(dkc2, dvc2)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(dkc2, dvc2)
    for rep in range(3):
        out.zero_(); pout["accept_len"].fill_(-7); cout["slot_map"].fill_(-7); mask_out["retrieve"].fill_(-7)
        dkc2.copy_(to_dev(kc)); dvc2.copy_(to_dev(vc))     # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        check(dkc2, dvc2, f"graph replay {rep}")


def test_full_step_headline_sweep_cell_as_a_replayed_graph():
    """The benchmark's default workload at full size (B = 32, P = 4096 paged, T = 128, depth 10, V = 32000; two layers
    instead of 32) in the launch configuration it times: tree tensors, attention per layer, fused epilogue, replayed as
    a HIP graph.  Every integer output and every cache byte against the oracle over the full batch; attention against
    the oracle on two seeded sequences per layer (all heads and rows; the full sweep of cells is in
    test_gpu_attention.py)."""
    L = 2
    wl = synth.config5(128, 10)
    rng = np.random.default_rng(98)
    q = np.stack([wl.q] + [synth._values(rng, wl.q.shape, "bf16") for _ in range(L - 1)])
    kt = np.stack([wl.kt] + [synth._values(rng, wl.kt.shape, "bf16") for _ in range(L - 1)])
    vt = np.stack([wl.vt] + [synth._values(rng, wl.vt.shape, "bf16") for _ in range(L - 1)])
    kc = np.stack([wl.k_cache] + [synth._values(rng, wl.k_cache.shape, "bf16") for _ in range(L - 1)])
    vc = np.stack([wl.v_cache] + [synth._values(rng, wl.v_cache.shape, "bf16") for _ in range(L - 1)])
    B, T, W, L_max = wl.B, wl.T_max, wl.W, wl.retrieve.shape[1]
    # oracle, integer path over the full batch
    rm = oracle.build_tree_mask(wl.parent, wl.n_nodes)
    rt = oracle.tensorize_tree(wl.parent, wl.n_nodes, wl.prefix_len, L_max, W)
    assert np.array_equal(rt["retrieve"], wl.retrieve) and (wl.retrieve < 0).mean() >= 0.5   # padding-heavy, as specified
    rg = oracle.safe_gather_paths(wl.retrieve, wl.n_nodes, T, 0, wl.tokens.reshape(B, T, 1))
    rp = oracle.evaluate_posterior(wl.logits, wl.tokens, wl.retrieve, wl.n_nodes)
    assert rp["accept_len"].tolist() == [a for _, a in wl.planted]
    rkc, rvc = kc.copy(), vc.copy()
    rc = oracle.commit_accepted_kv(kt, vt, rkc, rvc, wl.prefix_len, wl.capacity, wl.n_nodes, rp["acc_nodes"],
                                   rp["accept_len"], block_table=wl.block_table)
    assert np.all(rc["status"] == 0)

    d = DevWorkload(wl)
    dq, dkt, dvt, dkc, dvc = to_dev(q), to_dev(kt), to_dev(vt), to_dev(kc), to_dev(vc)
    out = torch.empty_like(dq)
    desc = api.attn_desc(dq[0], dkt[0], dkc[0], d.block_table, d.P_max)
    plan = api.tree_verify_attention_plan(desc)
    assert plan["mfma"] == 1 and plan["wavefronts"] == 8 and plan["n_splits"] == 1      # the shape bench.py reports
    ws = torch.empty(max(256, api.tree_verify_attention_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
    pws = torch.empty(max(256, api.evaluate_posterior_workspace_bytes(B, T, wl.V)), dtype=torch.uint8, device="cuda")
    holder = {}

    def step():
        m = api.tensorize_tree(d.parent, d.n_nodes, d.prefix_len, L_max, W, out=holder.get("m"))
        holder["m"] = m
        for l in range(L):
            api.tree_verify_attention(dq[l], dkc[l], dvc[l], d.prefix_len, dkt[l], dvt[l], m["bitmask"], d.n_nodes,
                                      P_max=d.P_max, block_table=d.block_table, out=out[l], want_lse=False,
                                      workspace=ws, desc=desc)
        holder["e"] = api.verify_epilogue(d.logits, d.tokens, m["retrieve"], d.n_nodes, dkt, dvt, dkc, dvc, d.prefix_len,
                                          d.capacity, block_table=d.block_table, src=d.tokens.reshape(B, T, 1),
                                          workspace=pws, gather_out=holder.get("g"), post_out=holder.get("p"),
                                          commit_out=holder.get("c"))
        holder["g"], holder["p"], holder["c"] = holder["e"]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                             # allocates the outputs once, outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    seqs = sorted(int(x) for x in np.random.default_rng(97).choice(B, size=2, replace=False))
    for rep in range(2):
        out.zero_(); holder["p"]["accept_len"].fill_(-7); holder["c"]["slot_map"].fill_(-7)
        dkc.copy_(to_dev(kc)); dvc.copy_(to_dev(vc))       # eager work between replays: the caches are committed into
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        m, g, p, c = holder["m"], holder["g"], holder["p"], holder["c"]
        assert np.array_equal(bits_of(m["dense"]), rm["dense"]) and np.array_equal(bits_of(m["status"]), rm["status"])
        for key in ("depth", "position_ids", "retrieve", "n_paths"):
            assert np.array_equal(bits_of(m[key]), rt[key]), (rep, key)
        for key in ("safe", "pvalid", "gathered"):
            assert np.array_equal(bits_of(g[key]), rg[key]), (rep, key)
        for key in rp:
            assert np.array_equal(bits_of(p[key]), rp[key]), (rep, key)
        for key in rc:
            assert np.array_equal(bits_of(c[key]), rc[key]), (rep, key)
        assert np.array_equal(bits_of(dkc), rkc) and np.array_equal(bits_of(dvc), rvc), rep
        for l in range(L):
            for b in seqs:
                sl = slice(b, b + 1)
                ref, _ = oracle.tree_verify_attention(q[l][sl], kc[l], vc[l], wl.prefix_len[sl], kt[l][sl], vt[l][sl],
                                                      rm["dense"][sl], wl.n_nodes[sl], dtype="bf16",
                                                      block_table=wl.block_table[sl], want_lse=False)
                err, rel, pz = attention_errors(out[l][sl], ref, wl.n_nodes[sl])
                assert pz and err <= 2e-2 and rel <= 2e-2, (rep, l, b, err, rel)
